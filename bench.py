#!/usr/bin/env python3
"""Benchmark of the fused CoCoDC sync step (cocodc_sync_step) on ONE MI355X.

A "step" is one pass of the whole path -- pseudo-gradient, outer Nesterov update, delay
compensation merge, fragment scores, fragment selection -- over every fragment of one
synthetic, model-shaped fragment set that is already resident in HBM.

Prints one JSON line: whole-job throughput in Gparams/s, the HBM roofline of the fused
element-wise kernel (algorithmic bytes / its HIP-event duration, measured in the same timed
region) and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak
BYTES_PER_PARAM = 36   # 5 fp32 reads + 4 fp32 writes (theta_m, theta_g, momentum, pseudo-gradient)

PROFILE_DIR = os.path.join(ROOT, "profiles")
KERNEL_SOURCES = ("paper_2504_17672_amd/csrc/cocodc_device.h", "paper_2504_17672_amd/csrc/cocodc.hip")


def kernel_source_sha256():
    """Fingerprint of the files that define the streaming kernels and their build switches."""
    import hashlib
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def profiled_traffic(workload, bf16):
    """HBM bytes per launch of the fused kernel as the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs recorded in
    profiles/fused_sync_step[_bf16]_<workload>.txt measured them (each counter scaled by what it reads for a plain
    device copy of known size; the summary names the commands).  The number belongs to the kernel sources it
    was measured on: the summary carries their fingerprint, and when the sources have changed since (or no
    summary exists for the workload) there is nothing to report: (None, reason)."""
    import re
    name = f"fused_sync_step_{'bf16_' if bf16 else ''}{workload}.txt"
    path = os.path.join(PROFILE_DIR, name)
    if not os.path.exists(path):
        return None, f"no profile summary profiles/{name}"
    text = open(path).read()
    m_hash = re.search(r"kernel_source_sha256:\s*([0-9a-f]{64})", text)
    m_traffic = re.search(r"traffic_bytes_per_launch:\s*(\d+)", text)
    if not m_hash or not m_traffic:
        return None, f"profiles/{name} carries no traffic figure"
    if m_hash.group(1) != kernel_source_sha256():
        return None, f"profiles/{name} was measured on other kernel sources"
    return int(m_traffic.group(1)), f"profiles/{name}"


def cpu_baseline(wl, st, bk, sample_frag, seconds_per_leg=6.0):
    """Times the oracle (as it stands) on one fragment of the workload, on the host cores: first on one
    thread, then chunk-parallel on all of them, each leg repeated for about seconds_per_leg (at least three
    runs); the best run of a leg counts, the median is reported beside it."""
    import numpy as np
    import oracle as ref
    off, ln = wl.frags[sample_frag]
    host0 = {k: v[off:off + ln].cpu().numpy().copy() for k, v in st.items()}
    frags = [(0, ln)]
    hp = ref.hparams(wl.tau, wl.H, wl.lam, wl.eta, wl.mu)
    I_p, t_b = [bk.I_p[sample_frag]], [bk.t_b[sample_frag]]
    pg = np.empty(ln, np.float32)

    def run(n_threads):
        times, used, spent = [], 1, 0.0
        while len(times) < 3 or (spent < seconds_per_leg and len(times) < 200):
            h = {k: v.copy() for k, v in host0.items()}
            t0 = time.perf_counter()
            out = ref.sync_step(frags, h["theta_m"], h["theta_m_send"], h["theta_g"], h["momentum"],
                                h["delta_g"], pg, I_p, t_b, bk.t_g, 1, hp, n_threads=n_threads)
            dt = time.perf_counter() - t0
            assert out["rc"] == 0
            used = out.get("threads", 1)
            times.append(dt)
            spent += dt
        times.sort()
        return times[0], times[len(times) // 2], len(times), used

    t1, t1_med, n1, _ = run(None)
    avail = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    env = os.environ.get("OMP_NUM_THREADS")
    want = min(avail, int(env)) if env and env.isdigit() else avail
    tm, tm_med, nm, used = run(max(1, want))
    return {
        "value": round(ln / tm / 1e9, 4), "unit": "Gparams/s", "cores": int(used), "kind": "oracle",
        "sample": f"fragment {sample_frag} of {wl.name} ({ln} params), fused oracle step, "
                  f"chunk-parallel over {used} threads, best of {nm} runs (median {ln / tm_med / 1e9:.3f}); "
                  f"single thread: best of {n1} runs (median {ln / t1_med / 1e9:.3f})",
        "single_thread_value": round(ln / t1 / 1e9, 4),
        "host_cpus_visible": avail,
    }


def placement_probe(B, torch, wl, dev):
    """Times the fused step (algorithmic GB/s, best of 3 launches after one warm-up) for many placements of
    the six buffers inside one allocation of 95 % of the free device memory.  Offsets are whole GiB from the
    start of that allocation; the buffer order is theta_m, theta_m_send, theta_g, momentum, delta_g, pg."""
    n, K, GiB = wl.n_total, wl.K, 1 << 30
    nb = 4 * n
    free, total = torch.cuda.mem_get_info(dev)
    arena_gib = int(free * 0.95) // GiB
    arena = torch.empty(arena_gib * GiB, dtype=torch.uint8, device=dev)
    for off in range(0, arena.numel(), 8 * GiB):
        arena[off:off + 8 * GiB].zero_()
    ws = B.new_workspace(K, n, dev)
    R = torch.zeros(K, dtype=torch.float64, device=dev)
    sel = torch.zeros(K, dtype=torch.int32, device=dev)
    n_sel = torch.zeros(1, dtype=torch.int32, device=dev)
    hp, ones = B.hparams(5, 100), [1] * K
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    b = (nb + GiB - 1) // GiB          # a buffer, in whole GiB
    top = arena_gib - b                # the last offset a buffer can start at

    def gbps(bases_gib):
        bases = sorted(int(o) * GiB for o in bases_gib)
        assert bases[0] >= 0 and bases[-1] + nb <= arena.numel() and all(x + nb <= y for x, y in zip(bases, bases[1:]))
        t = [arena[int(o) * GiB:int(o) * GiB + nb].view(torch.float32) for o in bases_gib]
        best = float("inf")
        for it in range(4):
            e0.record()
            B.check(B.cocodc_sync_step(wl.frags, n, t[0], t[1], t[2], t[3], t[4], t[5], ones, ones, 2, 1, hp, R, sel,
                                       n_sel, None, ws))
            e1.record()
            torch.cuda.synchronize()
            if it:
                best = min(best, e0.elapsed_time(e1))
        return round(36 * n / (best * 1e-3) / 1e9)

    step = 8 if b <= 8 else 10
    out = {"mode": "placement-probe", "workload": wl.name, "buffer_GiB": round(nb / GiB, 3),
           "device_memory_GiB": round(total / GiB, 2), "allocation_GiB": arena_gib,
           "unit": "algorithmic GB/s of the fused step; offsets in GiB from the start of the allocation"}
    out["all_six_back_to_back_from_X"] = {X: gbps([X + k * b for k in range(6)])
                                          for X in range(0, top - 5 * b + 1, step)}
    print("[bench] back to back done", file=sys.stderr, flush=True)
    out["five_back_to_back_from_0_and_pg_at_X"] = {X: gbps([0, b, 2 * b, 3 * b, 4 * b, X])
                                                   for X in range(5 * b, top + 1, step)}
    out["five_back_to_back_from_0_and_theta_m_at_X"] = {X: gbps([X, 0, b, 2 * b, 3 * b, 4 * b])
                                                        for X in range(5 * b, top + 1, step)}
    print("[bench] one buffer moved done", file=sys.stderr, flush=True)
    out["theta_m_theta_g_delta_g_from_0_and_the_other_three_from_X"] = {
        X: gbps([0, X, b, X + b, 2 * b, X + 2 * b]) for X in range(3 * b, top - 2 * b + 1, step)}
    out["uniform_stride_S"] = {S: gbps([k * S for k in range(6)]) for S in range(b, top // 5 + 1, 4)}
    print(json.dumps(out), flush=True)


def region_probe(B, torch, wl, dev):
    """Times every entry point that streams several buffers with each of its buffers in each third of the
    device memory (all 3^k assignments; for the fused step theta_m stays in the first third, the thirds being
    interchangeable), inside one allocation of 95 % of the free memory made first in the process.  Offsets
    assume that this allocation maps onto the memory from the bottom up (bench.py --placement-probe shows the
    steps where that predicts them).  Prints one JSON line: algorithmic GB/s per assignment, best first."""
    import itertools
    n, K, GiB = wl.n_total, wl.K, 1 << 30
    nb = 4 * n
    free, total = torch.cuda.mem_get_info(dev)
    start = total - free
    arena = torch.empty(int(free * 0.95) // GiB * GiB, dtype=torch.uint8, device=dev)
    for off in range(0, arena.numel(), 8 * GiB):
        arena[off:off + 8 * GiB].zero_()
    ws = B.new_workspace(K, n, dev)
    R = torch.zeros(K, dtype=torch.float64, device=dev)
    sel = torch.zeros(K, dtype=torch.int32, device=dev)
    n_sel = torch.zeros(1, dtype=torch.int32, device=dev)
    hp, ones, fr = B.hparams(5, 100), [1] * K, wl.frags
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    slot = (nb + GiB - 1) // GiB * GiB + GiB

    def buf(region, k):
        o = max(region * (96 << 30) - start, 0) + 2 * GiB + k * slot
        assert o + nb <= min((region + 1) * (96 << 30) - start, arena.numel())
        return arena[o:o + nb].view(torch.float32)

    def gbps(call, bpp, assign):
        bufs = [buf(r, sum(1 for j in range(i) if assign[j] == r)) for i, r in enumerate(assign)]
        best = float("inf")
        for it in range(4):
            e0.record()
            B.check(call(bufs))
            e1.record()
            torch.cuda.synchronize()
            if it:
                best = min(best, e0.elapsed_time(e1))
        return round(bpp * n / (best * 1e-3) / 1e9)

    entries = [
        ("cocodc_pseudograd + send-time record", "reads theta_g, theta_m; writes pg, theta_m_send", 16, 4, False,
         lambda b: B.cocodc_pseudograd(fr, n, b[0], b[1], b[2], b[3], ws)),
        ("cocodc_pseudograd", "reads theta_g, theta_m; writes pg", 12, 3, False,
         lambda b: B.cocodc_pseudograd(fr, n, b[0], b[1], b[2], None, ws)),
        ("cocodc_outer_nesterov", "theta_g in place, momentum in place, reads delta_g", 20, 3, False,
         lambda b: B.cocodc_outer_nesterov(fr, n, b[0], b[1], b[2], hp, ws)),
        ("cocodc_delay_compensate", "theta_m in place, reads theta_m_send, theta_g", 16, 3, False,
         lambda b: B.cocodc_delay_compensate(fr, n, b[0], b[1], b[2], hp, ws)),
        ("cocodc_sync_step", "theta_m in place, reads theta_m_send, theta_g in place, momentum in place, reads "
         "delta_g, writes pg", 36, 6, True,
         lambda b: B.cocodc_sync_step(fr, n, b[0], b[1], b[2], b[3], b[4], b[5], ones, ones, 2, 1, hp, R, sel, n_sel,
                                      None, ws)),
    ]
    out = {"mode": "region-probe", "workload": wl.name, "buffer_GiB": round(nb / GiB, 3),
           "unit": "algorithmic GB/s; an assignment lists the third (0, 1, 2) of the device memory of each buffer in "
                   "the order given", "entries": []}
    for name, order, bpp, k, first_fixed, call in entries:
        rows = []
        for assign in itertools.product(range(3), repeat=k):
            if first_fixed and assign[0] != 0:
                continue
            rows.append([gbps(call, bpp, assign), "".join(map(str, assign))])
        rows.sort(reverse=True)
        out["entries"].append({"entry": name, "buffers": order, "bytes_per_param": bpp, "by_assignment": rows})
        print(f"[bench] {name} done", file=sys.stderr, flush=True)
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="7B", help="tiny | 125M | 350M | 1.3B | 7B")
    ap.add_argument("--blocks-per-cu", type=int, default=None, help="launch-shape override (tuning)")
    ap.add_argument("--no-pg", action="store_true", help="skip the pseudo-gradient output (32 B/param)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--no-packed-pass", action="store_true",
                    help="skip the second timed pass with the buffers back to back (the 'packed_layout' object)")
    ap.add_argument("--merge-mode", default="dc", choices=["dc", "blend", "replace"],
                    help="dc: delay compensation (Eq. 8, default); blend: Streaming-DiLoCo merge (Eq. 3, "
                         "alpha 0.5, no send-time record: 32 B/param); replace: blocking-DiLoCo merge")
    ap.add_argument("--layout", default="tuned", choices=["tuned", "spaced", "packed", "compact", "regions"],
                    help="tuned: the six buffers are carved out of one allocation at the stride that a "
                         "short probe at set-up finds fastest; spaced: fixed stride "
                         "cocodc_layout_stride_bytes(); packed: six separate allocations; compact: back to "
                         "back in one allocation of their own size, the fastest of a few made after "
                         "temporary ballast allocations of different sizes (layout.compact_fast_buffers); "
                         "regions: each buffer in a chosen third of the device memory (--regions; "
                         "layout.region_buffers)")
    ap.add_argument("--regions", default="0,0,0,1,1,2",
                    help="with --layout regions: the third (0, 1, 2) of the device memory for theta_m, "
                         "theta_m_send, theta_g, momentum, delta_g and the pseudo-gradient buffer")
    ap.add_argument("--stride-gib", type=float, default=None, help="override the spaced-layout stride")
    ap.add_argument("--bf16", action="store_true",
                    help="bf16 local parameters, send-time record and pseudo-gradient, fp32 global state "
                         "(cocodc_sync_step_bf16, 28 B/param)")
    ap.add_argument("--graph", action="store_true",
                    help="record one step into a HIP graph and time replays (launch-bound small workloads); "
                         "the per-kernel HIP events are not available then, the roofline uses the whole step")
    ap.add_argument("--strided-shards", type=int, default=0, metavar="K",
                    help="shard the workload's layers into K strided fragments (shard k = layers k, k+K, ...; "
                         "Sec. 4.1) on a layer-ordered buffer and time cocodc_sync_step_segmented instead")
    ap.add_argument("--loop-steps", type=int, default=0, metavar="T",
                    help="instead of the fused-step benchmark, drive the Sec. 3.2 loop (cocodc_loop_step) for T "
                         "inner steps with one worker and the in-place send/receive buffer, and report the "
                         "time of its receive and send events")
    ap.add_argument("--primitives", action="store_true",
                    help="time the five single-step entry points (and their sum against the fused step) "
                         "instead of the headline metric; prints its own JSON line")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="instead of the benchmark, run 5 plain device copies of MIB mebibytes (a kernel "
                         "of known traffic, to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings) and exit")
    ap.add_argument("--placement-probe", action="store_true",
                    help="instead of the benchmark, time the fused step with the six buffers at many places of "
                         "one allocation that covers nearly all of the device memory (all back to back from X; "
                         "one buffer moved to X; two groups of three; uniform strides) and print one JSON line: "
                         "shows which parts of the memory a working set must touch to run fast")
    ap.add_argument("--region-probe", action="store_true",
                    help="instead of the benchmark, time the single-step entry points and the fused step with each "
                         "of their buffers in each third of the device memory and print one JSON line")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives are part of the path); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2504_17672_amd import binding as B
    from paper_2504_17672_amd import layout as L
    from paper_2504_17672_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.calibrate_copy:
        nbytes = args.calibrate_copy << 20
        src = torch.empty(nbytes // 4, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": True, "launches": 5, "bytes_read_per_launch": nbytes,
                          "bytes_written_per_launch": nbytes}), flush=True)
        return
    wl = synth.WORKLOADS[args.workload]
    K, n = wl.K, wl.n_total
    if args.placement_probe:
        placement_probe(B, torch, wl, dev)
        return
    if args.region_probe:
        region_probe(B, torch, wl, dev)
        return
    print(f"[bench] workload {wl.name}: K={K} n={n} resident {5 * 4 * n / 1e9:.1f} GB", file=sys.stderr, flush=True)
    layout, arena, bufs, probe = args.layout, None, None, {}
    stride = B.cocodc_layout_stride_bytes(n) if args.stride_gib is None else int(args.stride_gib * (1 << 30))
    if layout in ("spaced", "tuned"):
        try:
            if layout == "tuned" and args.stride_gib is None:
                arena, carved, stride, probe = L.tuned_spaced_buffers(
                    n, wl.frags, dev, verbose=lambda m: print("[bench] layout probe:", m, file=sys.stderr, flush=True))
            else:
                arena, carved = L.spaced_buffers(n, 6, dev, None if args.stride_gib is None else stride)
                stride = carved[1].data_ptr() - carved[0].data_ptr()
            names = ("theta_m", "theta_m_send", "theta_g", "momentum", "delta_g", "pg")
            bufs = dict(zip(names, carved))
        except torch.OutOfMemoryError:
            print("[bench] not enough free HBM for the spaced layout; using separate allocations",
                  file=sys.stderr, flush=True)
            layout = "packed"
    if layout == "regions":
        regions = tuple(int(x) for x in args.regions.split(","))
        assert len(regions) == 6 and all(0 <= r <= 2 for r in regions)
        arena, carved, offs = L.region_buffers(n, regions, dev)
        stride = 0
        bufs = dict(zip(("theta_m", "theta_m_send", "theta_g", "momentum", "delta_g", "pg"), carved))
    if layout == "compact":
        arena, carved, probe_compact = L.compact_fast_buffers(
            n, wl.frags, dev, verbose=lambda m: print("[bench] layout probe:", m, file=sys.stderr, flush=True))
        stride = carved[1].data_ptr() - carved[0].data_ptr()
        bufs = dict(zip(("theta_m", "theta_m_send", "theta_g", "momentum", "delta_g", "pg"), carved))
    st = synth.make_state(wl, dev, seed=0, buffers=bufs)
    bk = synth.bookkeeping(wl)
    if args.no_pg:
        pg = None
    else:
        pg = bufs["pg"] if bufs is not None else torch.empty(n, dtype=torch.float32, device=dev)
    R = torch.zeros(K, dtype=torch.float64, device=dev)
    sel = torch.full((K,), -1, dtype=torch.int32, device=dev)
    n_sel = torch.zeros(1, dtype=torch.int32, device=dev)
    ws = B.new_workspace(K, n, dev)
    mode = {"dc": 0, "blend": 1, "replace": 2}[args.merge_mode]
    hp = B.hparams(wl.tau, wl.H, wl.lam, wl.eta, wl.mu, merge_mode=mode, alpha=0.5)
    send = st["theta_m_send"] if mode == 0 else None
    if args.blocks_per_cu is not None:
        B.cocodc_set_blocks_per_cu(args.blocks_per_cu)
    torch.cuda.synchronize()

    if args.primitives:
        assert pg is not None and mode == 0, "--primitives times the default delay-compensation path with pg"
        fr, th = wl.frags, st

        def timed(fn, launches_per_call=1):
            for _ in range(args.warmup):
                fn()
            B.check(B.cocodc_profiler_enable(args.steps * launches_per_call))
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                fn()
            torch.cuda.synchronize()
            wall = (time.perf_counter() - t0) / args.steps * 1e3
            cnt, ms = B.cocodc_profiler_collect(args.steps * launches_per_call)
            B.cocodc_profiler_disable()
            assert cnt == args.steps * launches_per_call, cnt
            return wall, sum(ms) / args.steps

        calls = [
            ("cocodc_pseudograd", "k_walk<PseudoGradOp>", 12,
             lambda: B.check(B.cocodc_pseudograd(fr, n, th["theta_g"], th["theta_m"], pg, None, ws))),
            ("cocodc_pseudograd + send-time record", "k_walk<PseudoGradOp>", 16,
             lambda: B.check(B.cocodc_pseudograd(fr, n, th["theta_g"], th["theta_m"], pg, th["theta_m_send"], ws))),
            ("cocodc_outer_nesterov", "k_walk<OuterOp>", 20,
             lambda: B.check(B.cocodc_outer_nesterov(fr, n, th["theta_g"], th["momentum"], th["delta_g"], hp, ws))),
            ("cocodc_delay_compensate", "k_walk<MergeOp>", 16,
             lambda: B.check(B.cocodc_delay_compensate(fr, n, th["theta_m"], th["theta_m_send"], th["theta_g"], hp,
                                                       ws))),
            ("cocodc_fragment_scores", "k_walk<ScoreOp>", 4,
             lambda: B.check(B.cocodc_fragment_scores(fr, n, th["delta_g"], bk.I_p, 2, R, None, ws))),
        ]
        rows = []
        for name, kernel, bpp, fn in calls:
            wall, k_ms = timed(fn)
            rows.append({"entry": name, "kernel": kernel, "bytes_per_param": bpp, "ms_per_call": round(wall, 4),
                         "kernel_ms_avg": round(k_ms, 4), "achieved_GBps": round(bpp * n / (k_ms * 1e-3) / 1e9, 1),
                         "frac_of_peak": round(bpp * n / (k_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)})
            print(f"[bench] {rows[-1]}", file=sys.stderr, flush=True)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            B.check(B.cocodc_select_fragments(K, R, bk.t_b, bk.t_g, wl.H, wl.budget, sel, n_sel, ws))
        torch.cuda.synchronize()
        sel_ms = (time.perf_counter() - t0) / args.steps * 1e3

        # For scale: the same two reads and one write per element through torch's own element-wise
        # kernel on the same three buffers (what a plain 2-read-1-write stream gets on this GPU).
        def torch_ms(fn):
            for _ in range(args.warmup):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / args.steps
        ref_rows = []
        for name, bpp, fn in (
                ("torch.sub(theta_g, theta_m, out=pg)", 12, lambda: torch.sub(th["theta_g"], th["theta_m"], out=pg)),
                ("pg.copy_(theta_g)", 8, lambda: pg.copy_(th["theta_g"])),
                ("pg.fill_(0)", 4, lambda: pg.fill_(0.0))):
            ms = torch_ms(fn)
            ref_rows.append({"reference": name, "bytes_per_param": bpp, "ms": round(ms, 4),
                             "achieved_GBps": round(bpp * n / (ms * 1e-3) / 1e9, 1)})
            print(f"[bench] {ref_rows[-1]}", file=sys.stderr, flush=True)

        def five():
            calls[0][3](); calls[2][3](); calls[3][3](); calls[4][3]()
            B.check(B.cocodc_select_fragments(K, R, bk.t_b, bk.t_g, wl.H, wl.budget, sel, n_sel, ws))
        seq_wall, seq_k = timed(five, 4)
        mix_wall, mix_k = timed(lambda: B.check(B.cocodc_debug_stream_mix(
            fr, n, th["theta_m"], th["theta_m_send"], th["theta_g"], th["momentum"], th["delta_g"], pg, ws)), 1)
        for name in ("theta_m", "theta_g", "momentum"):   # the additions above grew them; back to model scale
            th[name].normal_(0.0, 0.02)
        fused_wall, fused_k = timed(lambda: B.check(B.cocodc_sync_step(
            fr, n, th["theta_m"], th["theta_m_send"], th["theta_g"], th["momentum"], th["delta_g"], pg, bk.I_p,
            bk.t_b, bk.t_g, wl.budget, hp, R, sel, n_sel, None, ws)))
        assert bool(torch.isfinite(th["theta_m"][:1 << 20]).all().item())
        print(json.dumps({"mode": "primitives", "workload": wl.name, "params": n, "steps": args.steps,
                          "layout": layout + (" " + args.regions if layout == "regions" else ""),
                          "stride_GiB": round(stride / (1 << 30), 2), "entries": rows,
                          "select_ms_per_call": round(sel_ms, 4), "torch_references": ref_rows,
                          "five_calls_in_sequence": {"bytes_per_param": 52, "ms": round(seq_wall, 4),
                                                     "Gparams_per_s": round(n / seq_wall / 1e6, 2)},
                          "same_streams_no_arithmetic": {
                              "entry": "cocodc_debug_stream_mix", "bytes_per_param": 36, "kernel_ms_avg": round(mix_k, 4),
                              "achieved_GBps": round(36 * n / (mix_k * 1e-3) / 1e9, 1),
                              "fused_kernel_ms_avg": round(fused_k, 4),
                              "fused_kernel_over_this": round(fused_k / mix_k, 4)},
                          "fused": {"bytes_per_param": 36, "ms": round(fused_wall, 4),
                                    "Gparams_per_s": round(n / fused_wall / 1e6, 2),
                                    "speedup_over_sequence": round(seq_wall / fused_wall, 3)}}), flush=True)
        return

    cpu = None
    if not args.no_cpu and not args.bf16 and not args.loop_steps:  # the timed CPU oracle is the fp32 step
        sample = 1 if K > 1 else 0
        print(f"[bench] timing the CPU oracle on fragment {sample}", file=sys.stderr, flush=True)
        cpu = cpu_baseline(wl, st, bk, sample)
        print(f"[bench] cpu baseline {cpu}", file=sys.stderr, flush=True)

    if args.bf16:
        # same placement: each bf16 buffer occupies the first half of its fp32-sized slot
        # converted in place, chunk by chunk in ascending order: a converted chunk always lies below
        # the fp32 chunk it came from, so no source element is overwritten before it is read
        for name in ("theta_m", "theta_m_send"):
            src = st[name]
            dst = src.view(torch.bfloat16)
            for lo in range(0, n, 1 << 28):
                hi = min(n, lo + (1 << 28))
                dst[lo:hi].copy_(src[lo:hi].to(torch.bfloat16))  # dst[lo:hi] lies below src[lo:hi]: safe ascending
            st[name] = dst[:n]
        if pg is not None:
            pg = pg.view(torch.bfloat16)[:n]
        send = st["theta_m_send"] if mode == 0 else None

    if args.loop_steps:
        lens = [l for _, l in wl.frags]
        if args.strided_shards:   # the paper's partition: shard k = layers k, k + K, ... (Sec. 4.1)
            assert wl.model, "--strided-shards needs a model-shaped workload"
            lsegs, n_seg = synth.strided_segments(*wl.model, args.strided_shards)
            assert n_seg == n
            K = args.strided_shards
            lens = [sum(l for _, l, f in lsegs if f == p) for p in range(K)]
            R = torch.zeros(K, dtype=torch.float64, device=dev)
            sel = torch.full((K,), -1, dtype=torch.int32, device=dev)
            ws = B.new_workspace_segmented(len(lsegs), K, n, dev)
            rc, loop = B.cocodc_loop_create_segmented(lsegs, K, n, hp, 1.0, 1.0, float(wl.tau))
        else:
            rc, loop = B.cocodc_loop_create(wl.frags, n, hp, 1.0, 1.0, float(wl.tau))  # T_s = tau * T_c
        B.check(rc)
        B.check(B.cocodc_loop_reset_scores(loop, R))
        if args.bf16:   # the arriving average is fp32, the outgoing pseudo-gradient 16-bit: two buffers
            assert pg is not None, "the bf16 loop needs the send buffer"
            loop_step, send_buf = B.cocodc_loop_step_bf16, pg
            rec_bytes, snd_bytes = 26, 10
        else:           # one worker, closed loop: the pseudo-gradient is written over delta_g
            loop_step, send_buf = B.cocodc_loop_step, st["delta_g"]
            rec_bytes, snd_bytes = 32, 16
        lb = B.loop_buffers(st["theta_m"], st["theta_m_send"], st["theta_g"], st["momentum"], st["delta_g"],
                            send_buf, R, sel, n_sel, ws)
        _, N_plan, h_plan = B.cocodc_loop_plan(loop)
        ev, host_s = [], 0.0
        B.check(B.cocodc_profiler_enable(2 * args.loop_steps + 8))   # HIP events around the two streaming kernels
        torch.cuda.synchronize()
        t_all = time.perf_counter()
        for t in range(1, args.loop_steps + 1):
            t0 = time.perf_counter()
            rc, rec, sent = loop_step(loop, t, lb)
            B.check(rc)
            host_s += time.perf_counter() - t0   # the call itself never waits for the stream
            if rec or sent == B.COCODC_LOOP_SENT_PENDING:
                torch.cuda.synchronize()         # the benchmark's own wait, to time the event on the GPU
                dt = time.perf_counter() - t0
                if sent == B.COCODC_LOOP_SENT_PENDING:
                    sent = B.cocodc_loop_last_sent(loop)[2]
                ev.append((dt, rec, sent))
        torch.cuda.synchronize()
        t_all = time.perf_counter() - t_all
        B.cocodc_loop_destroy(loop)
        n_k, k_ms = B.cocodc_profiler_collect(2 * args.loop_steps + 8)
        B.cocodc_profiler_disable()
        # kernel durations in launch order: per event the fused step on the arrived fragments (if any arrived and
        # are not empty), then the walk over the chosen fragment (if one was chosen and is not empty)
        it_ms, rec_k, snd_k = iter(k_ms[:max(n_k, 0)]), [0, 0.0], [0, 0.0]
        for _, rec, snt in ev:
            if sum(lens[p] for p in rec) > 0:
                rec_k[0] += sum(lens[p] for p in rec)
                rec_k[1] += next(it_ms, 0.0)
            if snt >= 0 and lens[snt] > 0:
                snd_k[0] += lens[snt]
                snd_k[1] += next(it_ms, 0.0)
        rec_p = sum(lens[p] for _, rec, _ in ev for p in rec)
        snd_p = sum(lens[s] for _, _, s in ev if s >= 0)
        only_rec = [(dt, sum(lens[p] for p in rec)) for dt, rec, s in ev if rec and s < 0]
        only_snd = [(dt, lens[s]) for dt, rec, s in ev if not rec and s >= 0]
        out = {"mode": "loop", "workload": wl.name, "inner_steps": args.loop_steps, "tau": wl.tau, "H": wl.H, "K": K,
               "fragments": f"{K} strided shards" if args.strided_shards else "contiguous",
               "N": N_plan, "h": h_plan, "events": len(ev), "received_params": rec_p, "sent_params": snd_p,
               "loop_seconds": round(t_all, 4), "host_seconds_inside_loop_step": round(host_s, 4),
               "receive_Gparams_per_s": round(sum(p for _, p in only_rec) / max(sum(d for d, _ in only_rec), 1e-12) / 1e9, 2),
               "send_Gparams_per_s": round(sum(p for _, p in only_snd) / max(sum(d for d, _ in only_snd), 1e-12) / 1e9, 2),
               "receive_kernel_GBps": round(rec_bytes * rec_k[0] / max(rec_k[1], 1e-9) / 1e6, 1),
               "send_kernel_GBps": round(snd_bytes * snd_k[0] / max(snd_k[1], 1e-9) / 1e6, 1),
               "dtype": "bf16 local parameters, fp32 global state" if args.bf16 else "f32",
               "receive_bytes_per_param": rec_bytes, "send_bytes_per_param": snd_bytes,
               "all_events_GBps": round(sum(rec_bytes * sum(lens[p] for p in rec) + (snd_bytes * lens[s] if s >= 0 else 0)
                                            for _, rec, s in ev) / max(sum(d for d, _, _ in ev), 1e-12) / 1e9, 1)}
        print(json.dumps(out), flush=True)
        return

    segs = None
    if args.strided_shards:
        assert wl.model, "--strided-shards needs a model-shaped workload"
        segs, n_seg = synth.strided_segments(*wl.model, args.strided_shards)
        assert n_seg == n
        Ks = args.strided_shards
        h = max(1, wl.H // Ks)
        I_s = [h * (1 + p % 3) for p in range(Ks)]
        tb_s = [bk.t_g - i for i in I_s]
        ws = B.new_workspace_segmented(len(segs), Ks, n, dev)

    def step():
        if args.bf16:
            B.check(B.cocodc_sync_step_bf16(wl.frags, n, st["theta_m"], send, st["theta_g"], st["momentum"],
                                            st["delta_g"], pg, bk.I_p, bk.t_b, bk.t_g, wl.budget, hp, R, sel, n_sel,
                                            None, ws))
            return
        if segs is not None:
            B.check(B.cocodc_sync_step_segmented(segs, Ks, n, st["theta_m"], send, st["theta_g"], st["momentum"],
                                                 st["delta_g"], pg, I_s, tb_s, bk.t_g, min(wl.budget, Ks), hp, R, sel,
                                                 n_sel, None, ws))
            return
        B.check(B.cocodc_sync_step(wl.frags, n, st["theta_m"], send, st["theta_g"], st["momentum"],
                                   st["delta_g"], pg, bk.I_p, bk.t_b, bk.t_g, wl.budget, hp, R, sel, n_sel, None,
                                   ws))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.graph:
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.graph(graph, stream=side):
            step()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        k1_ms = [elapsed / args.steps * 1e3] * args.steps
    else:
        B.check(B.cocodc_profiler_enable(args.steps))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        cnt, k1_ms = B.cocodc_profiler_collect(args.steps)
        B.cocodc_profiler_disable()
        assert cnt == args.steps, cnt
    finite = bool(torch.isfinite(st["theta_m"][:1 << 20]).all().item())
    assert finite, "state went non-finite during the timed steps"

    ms_per_step = elapsed / args.steps * 1e3
    k1_avg = sum(k1_ms) / len(k1_ms)
    bpp = BYTES_PER_PARAM - (4 if args.no_pg else 0) - (4 if mode != 0 else 0)
    if args.bf16:  # theta_m read+written, theta_m_send read, pseudo-gradient written: 2 bytes each
        bpp = (2 + 4 + 4 + 4 + (2 if mode == 0 else 0)) + (2 + 4 + 4 + (0 if args.no_pg else 2))
    achieved = bpp * n / (k1_avg * 1e-3) / 1e9
    selected = sel[:int(n_sel.item())].cpu().tolist()

    # What the placement is worth.  (a) The set-up probe timed the fused step at every candidate
    # stride: which is the smallest arena that still reaches 80 % of the HBM peak?  (b) The same
    # timed region once more with the six buffers back to back in the same allocation, which is
    # where separate hipMalloc calls put them.
    GiB = 1 << 30
    nbytes = 4 * n
    layout_detail = {"kind": layout}
    if layout == "regions":
        layout_detail.update(regions=list(regions), offsets_GiB=[round(o / GiB, 2) for o in offs],
                             arena_GiB=round(arena.numel() / GiB, 1))
    elif arena is not None:
        layout_detail.update(stride_GiB=round(stride / GiB, 2), arena_GiB=round(arena.numel() / GiB, 1),
                             used_span_GiB=round((5 * stride + nbytes) / GiB, 1))
    if layout == "compact":
        layout_detail["probe_GBps_by_ballast_GiB"] = {f"{g:g}": v for g, v in probe_compact.items()}
    if probe:
        gbps = {g: 36 * n / (ms * 1e-3) / 1e9 for g, ms in probe.items()}
        layout_detail["probe_GBps_by_stride_GiB"] = {f"{g:g}": round(v, 0) for g, v in sorted(gbps.items())}
        ok = [g for g, v in sorted(gbps.items()) if v >= 0.8 * HBM_PEAK_GBS]
        layout_detail["smallest_stride_GiB_with_80pct"] = ok[0] if ok else None
        layout_detail["span_GiB_at_that_stride"] = round((5 * ok[0] * GiB + nbytes) / GiB, 1) if ok else None
    packed = None
    plain = (arena is not None and not args.graph and not args.bf16 and segs is None and mode == 0 and pg is not None)
    if plain and not args.no_packed_pass and layout not in ("compact", "regions"):   # (compact is back to back itself)
        pstride = (nbytes + 255) // 256 * 256
        pviews = [arena[k * pstride:k * pstride + nbytes].view(torch.float32) for k in range(6)]
        pbufs = dict(zip(("theta_m", "theta_m_send", "theta_g", "momentum", "delta_g", "pg"), pviews))
        del st
        pst = synth.make_state(wl, dev, seed=0, buffers=pbufs)   # overwrites the tuned buffers: they are done
        ppg = pbufs["pg"]

        def pstep():
            B.check(B.cocodc_sync_step(wl.frags, n, pst["theta_m"], pst["theta_m_send"], pst["theta_g"],
                                       pst["momentum"], pst["delta_g"], ppg, bk.I_p, bk.t_b, bk.t_g, wl.budget, hp, R,
                                       sel, n_sel, None, ws))
        for _ in range(args.warmup):
            pstep()
        B.check(B.cocodc_profiler_enable(args.steps))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            pstep()
        torch.cuda.synchronize()
        p_elapsed = time.perf_counter() - t0
        cnt, p_ms = B.cocodc_profiler_collect(args.steps)
        B.cocodc_profiler_disable()
        assert cnt == args.steps
        p_avg = sum(p_ms) / len(p_ms)
        p_ach = bpp * n / (p_avg * 1e-3) / 1e9
        packed = {"layout": "the six buffers back to back in one allocation (what separate allocations give)",
                  "span_GiB": round(6 * pstride / GiB, 1), "value": round(n / (p_elapsed / args.steps) / 1e9, 3),
                  "unit": "Gparams/s", "ms_per_step": round(p_elapsed / args.steps * 1e3, 4),
                  "kernel_ms_avg": round(p_avg, 4), "achieved": round(p_ach, 1),
                  "frac": round(p_ach / HBM_PEAK_GBS, 4)}
    traffic, traffic_source = (None, "not the profiled configuration")
    if mode == 0 and not args.no_pg and segs is None and not args.graph:
        traffic, traffic_source = profiled_traffic(wl.name, args.bf16)
    out = {
        "metric": "fused sync-step Gparams/s and achieved HBM GB/s (% of peak), 1\u00d7MI355X",
        "value": round(n / (elapsed / args.steps) / 1e9, 3),
        "unit": "Gparams/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": wl.name, "K": K, "params": n, "tau": wl.tau, "H": wl.H, "budget": wl.budget,
                   "bytes_per_param": bpp, "merge_mode": args.merge_mode,
                   "arithmetic": "fp64 in registers, each stored value rounded once",
                   "storage_dtype": "bf16 local parameters, f32 global state" if args.bf16 else "f32",
                   "launch": "hip graph replay" if args.graph else "eager",
                   "fragments": (f"{args.strided_shards} strided shards of {len(segs)} segments" if segs
                                 else "contiguous"),
                   "layout": ("packed: separate allocations" if layout == "packed" else
                              f"regions: one allocation, the buffers in thirds {args.regions} of the device memory"
                              if layout == "regions" else
                              f"{layout}: one allocation, buffer bases {stride / (1 << 30):.2f} GiB apart"),
                   "layout_detail": layout_detail,
                   "selected": selected},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": "k_walk<FusedBf16Op>" if args.bf16 else "k_walk<FusedOp>", "kernel_ms_avg": round(k1_avg, 4),
                     "kernel_ms_min": round(min(k1_ms), 4), "algorithmic_bytes": bpp * n},
        "packed_layout": packed,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
