"""Throughput of AdaComp's data-parallel hot path on one MI355X.

Workload ("flat", the roofline configuration): a stream of 1B-element fp32 gradients in
100 tensors of 10M, mixture 95% N(0,1e-5) + 5% N(0,1e-2), rate 0.5% per tensor, 16
queued worker updates with staleness uniform in [1,16].  One step = one pass of the
whole path over one batch of 16 worker gradients, all resident in HBM: adacomp_select
over all of them (one call over the 1600 tensors by default, or 16 calls with
--per-gradient-calls), then one adacomp_apply of the 16-update queue.  Three such batches
(48 distinct worker gradients, 192 GB) stay resident and step i works on batch i mod 3: the
stream is not one batch selected over and over, and the buffers span most of the HBM (the
filter's speed depends on where its input lies, see profiles/filter_placement.md).  For the
same reason the run waits 20 s before it touches the GPU (--settle): buffers allocated within
seconds of another process releasing as many land differently in the card's memory and are
read 7 % slower for the life of the process (profiles/filter_after_idle.md).
value = gradient elements compressed and applied per second = 16e9 / step time.

--workload paper_cnn runs the same step on the network size and worker count of the paper's own
experiments (211,690 parameters, 200 workers): a latency regime, reported the same way.

Prints ONE JSON line.  `roofline` is for the dominant kernel (select's streaming filter
pass), timed live with HIP events on the launch stream inside the timed steps;
`roofline_apply` is the same for the apply's kernels, `whole_path` prices the whole step
by its algorithmic bytes, `per_gradient_calls` times the same step with one select call per
worker gradient, `copy_ceiling_GBps` is what a plain device copy reaches on the same box;
`cpu_baseline` is the CPU oracle as it stands on a bounded sample, on all host cores of
the box's share (one tensor per thread) with the single-thread figure beside it.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def cpu_baseline(cfg, rate, lr, pulls, n_updates=8):
    """Oracle select + apply of `n_updates` worker updates.  flat: on one 10M-entry tensor with one
    thread, then on one tensor per thread with all cores of the box's share (tensors are independent
    in both halves of the method); other workloads: the whole model, one thread."""
    from concurrent.futures import ThreadPoolExecutor

    import oracle
    import workloads

    def run(layers, n_up):
        grads = [[workloads.gradient_layer(cfg, q, l).numpy() for l in layers] for q in range(n_up)]
        theta = [t.numpy().copy() for t in workloads.theta0(cfg, layers=layers)]
        ps = oracle.ParameterServer(theta)
        t0 = time.perf_counter()
        for q in range(n_up):
            off, idx, val = oracle.select(grads[q], rate)
            ps.apply(off, idx, val, min(pulls[q], q), lr)
        return time.perf_counter() - t0, n_up * sum(g.size for g in grads[0])

    whole = cfg != "flat"
    if whole:     # about 1.6e8 elements through the oracle: 10 to 20 s
        layers = list(range(len(workloads.sizes_of(cfg))))
        n_updates = max(1, min(len(pulls), int(1.6e8 // sum(workloads.sizes_of(cfg)))))
        print(f"[bench] cpu baseline: oracle on {n_updates} updates, 1 thread", file=sys.stderr, flush=True)
        dt, elems = run(layers, n_updates)
        return {"value": elems / dt, "unit": "elements/s", "cores": 1, "kind": "oracle",
                "sample": f"{n_updates} worker updates of the whole model of the {cfg} workload "
                          f"(select at {rate}, then PS apply), {dt:.1f} s of single-thread C"}
    print(f"[bench] cpu baseline: oracle on {n_updates} updates of one tensor, 1 thread", file=sys.stderr, flush=True)
    dt1, elems1 = run([0], n_updates)
    cores = max(1, min(os.cpu_count() or 1, 16))     # the machine's CPU share for one GPU
    print(f"[bench] cpu baseline: the same on {cores} tensors, one per thread", file=sys.stderr, flush=True)
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as ex:     # the C calls release the GIL
        parts = list(ex.map(lambda l: run([l], n_updates), range(cores)))
    dtc = time.perf_counter() - t0                        # includes generating the inputs: counted against the oracle
    busy = max(p[0] for p in parts)
    elems = sum(p[1] for p in parts)
    return {"value": elems / busy, "unit": "elements/s", "cores": cores, "kind": "oracle",
            "sample": f"{n_updates} worker updates of {cores} of the 100 10M-entry tensors of the flat workload, one tensor per "
                      f"thread (select at {rate}, then PS apply): {busy:.1f} s in the slowest thread ({dtc:.1f} s with input "
                      f"generation); one thread on one tensor: {elems1 / dt1:.3e} elements/s in {dt1:.1f} s",
            "single_thread_value": elems1 / dt1}


def gpu_state(step, torch, busy_s=1.2, samples=4):
    """Clocks, power and temperature of the card as rocm-smi reads them while untimed steps keep it busy:
    the same binary runs a few per cent faster or slower from one box (one physical GPU) to the next."""
    import subprocess
    t_end = time.perf_counter() + busy_s
    reads = []
    while time.perf_counter() < t_end:
        for _ in range(8):
            step()          # asynchronous: the queue stays a few steps deep
        try:
            r = subprocess.run(["rocm-smi", "--showclocks", "--showpower", "--showtemp", "--json"],
                               capture_output=True, text=True, timeout=20)
            card = next(iter(json.loads(r.stdout).values()))
            reads.append(card)
        except Exception:       # no rocm-smi, or output it cannot parse: the figure is context only
            break
        torch.cuda.synchronize()
        if len(reads) >= samples:
            break
    torch.cuda.synchronize()
    if not reads:
        return None

    def num(text):
        m = re.search(r"-?\d+(\.\d+)?", str(text))
        return float(m.group(0)) if m else None

    out = {"samples": len(reads), "sampled_during": "untimed steps after the timed region"}
    for key, name in (("sclk clock speed:", "sclk_MHz"), ("mclk clock speed:", "mclk_MHz"),
                      ("Temperature (Sensor junction) (C)", "junction_C"), ("Temperature (Sensor memory) (C)", "memory_C")):
        vals = [num(c.get(key)) for c in reads if num(c.get(key)) is not None]
        if vals:
            out[name] = {"min": min(vals), "max": max(vals)}
    for c in reads:
        for key, val in c.items():
            if "ower" in key and "(W)" in key and num(val) is not None:
                out.setdefault("power_W", {"min": num(val), "max": num(val)})
                out["power_W"]["min"] = min(out["power_W"]["min"], num(val))
                out["power_W"]["max"] = max(out["power_W"]["max"], num(val))
    return out


def placement_experiment(ac, workloads, torch, dev, n_sets, rounds=3, steps=8):
    """Same process, same call, different allocations: filter milliseconds per select call of 16e9 elements."""
    cfg, rate, Q = "flat", 0.005, 16
    sizes = workloads.sizes_of(cfg)
    L = len(sizes)
    cap = sum(ac.adacomp_count(n, rate) for n in sizes)
    ws = torch.empty(ac.adacomp_select_workspace(sizes * Q, rate), dtype=torch.uint8, device=dev)
    big = ac.Update(L * Q, cap * Q, dev)
    sets = []
    for i in range(n_sets):
        grads = [workloads.gradient(cfg, 100 * i + q, device=dev) for q in range(Q)]
        sets.append(ac.Layers([t for g in grads for t in g]))
    res = []
    for rnd in range(rounds):
        for i, layers in enumerate(sets):
            for _ in range(2):
                ac.adacomp_select(layers, rate, big, ws)
            torch.cuda.synchronize()
            ac.adacomp_profile_start({"filter"})
            for _ in range(steps):
                ac.adacomp_select(layers, rate, big, ws)
            torch.cuda.synchronize()
            ms, launches = ac.adacomp_profile_stop()["filter"]
            res.append({"round": rnd, "set": i, "filter_ms_per_call": ms / steps, "filter_launches_per_call": launches // steps})
    print(json.dumps({"experiment": "placement", "sets": n_sets, "elements_per_call": Q * sum(sizes), "results": res}), flush=True)


def view_offset_experiment(ac, torch, dev, n=400_000_000, rate=0.005, reps=5):
    """One tensor of n elements as a view that starts 0, 1, 2, 3, 8 and 33 elements into a buffer: select and filter time."""
    gen = torch.Generator(device=dev).manual_seed(3)
    base = torch.randn(n + 64, generator=gen, device=dev)
    k = ac.adacomp_count(n, rate)
    upd = ac.Update(1, k, dev)
    ws = torch.empty(ac.adacomp_select_workspace([n], rate), dtype=torch.uint8, device=dev)
    res = []
    for shift in (0, 1, 2, 3, 8, 33):
        layers = ac.Layers([base[shift:shift + n]])
        for _ in range(2):
            ac.adacomp_select(layers, rate, upd, ws)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ac.adacomp_profile_start({"filter"})
        e0.record()
        for _ in range(reps):
            ac.adacomp_select(layers, rate, upd, ws)
        e1.record()
        torch.cuda.synchronize()
        ms, _ = ac.adacomp_profile_stop()["filter"]
        res.append({"offset_elements": shift, "offset_bytes": 4 * shift, "select_us": 1e3 * e0.elapsed_time(e1) / reps,
                    "filter_us": 1e3 * ms / reps})
    print(json.dumps({"experiment": "view offset", "elements": n, "rate": rate, "results": res}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--breakdown", action="store_true", help="also time every kernel in one extra untimed step")
    ap.add_argument("--per-gradient-calls", action="store_true",
                    help="one adacomp_select call per worker gradient instead of one call over all 16")
    ap.add_argument("--streams", type=int, default=1,
                    help="HIP streams the 16 independent selects of a step are spread over (each has its own workspace)")
    ap.add_argument("--workload", default="flat", choices=["flat", "paper_cnn", "cnn_apply", "mid"],
                    help="flat: the roofline configuration (default, the one the metric is quoted on); paper_cnn: the "
                         "211,690-parameter network and 200 workers of the paper's experiments (latency regime); "
                         "cnn_apply, mid: the small and the mid-size CNN configurations")
    ap.add_argument("--rate", type=float, default=None, help="compression ratio c (default: the workload's first)")
    ap.add_argument("--rows-shared", action="store_true",
                    help="with --row-spread: the same rows are large in every worker's gradient")
    ap.add_argument("--row-spread", type=float, default=0.0,
                    help="scale every row of 1024 consecutive gradient elements by exp(s * N(0,1)): large entries "
                         "cluster in rows as in real weight gradients (default 0: the independent entries of the "
                         "named workload)")
    ap.add_argument("--graph", action="store_true",
                    help="record one step in a HIP graph and time replays of it (the kernel timing for `roofline` then "
                         "comes from the same number of eager steps run afterwards)")
    ap.add_argument("--wire", action="store_true",
                    help="also encode / decode one worker update in the wire format and report bytes and times")
    ap.add_argument("--no-copy-ceiling", action="store_true", help="skip the plain 4 GB device copy (flat workload)")
    ap.add_argument("--no-gpu-state", action="store_true", help="skip the rocm-smi readings under load (flat workload)")
    ap.add_argument("--batches", type=int, default=None,
                    help="distinct batches of worker gradients kept resident; step i works on batch i mod this (default: 3 for "
                         "flat = 48 gradients, 192 GB, so that the stream is not one batch selected over and over; 1 otherwise)")
    ap.add_argument("--placement-sets", type=int, default=0,
                    help="instead of the benchmark: allocate this many sets of 16 flat gradients (64 GB each) in one process, "
                         "time the same select call on each set in turn, three rounds, and print the filter time per set: "
                         "shows how much of the filter's run-to-run spread belongs to where the buffers lie in memory")
    ap.add_argument("--view-offsets", action="store_true",
                    help="instead of the benchmark: select on one 400M-element tensor that starts 0 to 33 elements into its "
                         "buffer (a view into a flat parameter buffer), time per call and of the filter")
    ap.add_argument("--no-per-gradient", action="store_true",
                    help="skip the extra steps with one select call per worker gradient (flat workload)")
    ap.add_argument("--settle", type=float, default=None,
                    help="seconds to wait before anything touches the GPU (default: 20 for flat, 0 otherwise). A process "
                         "that allocates its 200 GB within seconds of another one releasing as much gets them placed "
                         "differently in the card's memory, and the streaming read is then 7 %% slower for the life of "
                         "the process; after 20 s of idle the placement is that of a fresh machine")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")
    settle_s = args.settle if args.settle is not None else (20.0 if args.workload == "flat" else 0.0)
    if settle_s > 0:
        print(f"[bench] idling {settle_s:g} s before the first GPU allocation (--settle)", file=sys.stderr, flush=True)
        time.sleep(settle_s)

    import torch

    import paper_1702_04683_amd as ac
    import workloads

    ac.load_library()   # raises if libadacomp.so is not built: there is no fallback path
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dev = torch.device("cuda:0")
    cfg = args.workload
    c = workloads.CONFIGS[cfg]
    rate, lr, Q = (c["rates"][0] if args.rate is None else args.rate), c["lr"], c["Q"]
    small = cfg == "paper_cnn"      # every tensor is selected by one workgroup (k_small), not streamed by k_filter
    sizes = workloads.sizes_of(cfg)
    L, N = len(sizes), sum(sizes)
    pulls = workloads.pull_timestamps(workloads.staleness(cfg))

    if args.placement_sets > 0:
        placement_experiment(ac, workloads, torch, dev, args.placement_sets)
        return
    if args.view_offsets:
        view_offset_experiment(ac, torch, dev)
        return

    nb = args.batches if args.batches else (3 if cfg == "flat" else 1)
    # batch b holds the gradients of workers b*Q .. b*Q + Q-1 of the seeded stream: 16 x 4 GB resident per batch of flat
    batches = [[workloads.gradient(cfg, b * Q + q, device=dev, row_spread=args.row_spread, rows_shared=args.rows_shared)
                for q in range(Q)] for b in range(nb)]
    grads = batches[0]
    step_no = [0]
    theta = workloads.theta0(cfg, device=dev)
    state = ac.State(theta)
    cap = sum(ac.adacomp_count(n, rate) for n in sizes)
    updates = [ac.Update(L, cap, dev) for _ in range(Q)]
    batched = not args.per_gradient_calls
    ns = 1 if batched else max(1, args.streams)
    streams = [torch.cuda.Stream(device=dev) for _ in range(ns)] if ns > 1 else [torch.cuda.current_stream(dev)]
    sel_wss = []
    if not batched:
        sel_bytes = ac.adacomp_select_workspace(sizes, rate)
        sel_wss = [torch.empty(sel_bytes, dtype=torch.uint8, device=dev) for _ in range(ns)]
    if not batched:
        for q in range(Q):      # fills layer_off so that the apply workspace can be sized
            ac.adacomp_select(grads[q], rate, updates[q], sel_wss[q % ns])
    else:
        # the C ABI takes any list of tensors: all 16 worker gradients (1600 tensors) go through ONE
        # select call, so the small per-call kernels are paid once; its output buffers are then
        # viewed as the 16 worker updates (100 tensors each, own pull timestamp) that apply takes
        all_tensors_of = [ac.Layers([t for g in bt for t in g]) for bt in batches]     # marshalled once
        all_tensors = all_tensors_of[0]
        big = ac.Update(L * Q, cap * Q, dev)
        sel_wss = [torch.empty(ac.adacomp_select_workspace(sizes * Q, rate), dtype=torch.uint8, device=dev)]
        ac.adacomp_select(all_tensors, rate, big, sel_wss[0])
        updates = [big.view(q * L, (q + 1) * L) for q in range(Q)]
    app_ws = torch.empty(max(256, ac.adacomp_apply_workspace(sizes, updates)), dtype=torch.uint8, device=dev)
    params = ac.Layers(theta)          # marshalled once, like the queue
    queue = ac.Queue(updates)
    torch.cuda.synchronize()

    main = torch.cuda.current_stream(dev)

    def selects():
        t0 = state.t
        b = step_no[0] % nb        # the batch of worker gradients this step works on
        step_no[0] += 1
        if batched:
            for q in range(Q):
                updates[q].pull_ts = t0 + pulls[q]
            ac.adacomp_select(all_tensors_of[b], rate, big, sel_wss[0])
            return
        # the 16 worker updates are independent: spread them over the streams, then join
        if ns > 1:
            ready = main.record_event()
            for st in streams:
                st.wait_event(ready)        # the previous apply has consumed the update buffers
        for q in range(Q):
            updates[q].pull_ts = t0 + pulls[q]
            ac.adacomp_select(batches[b][q], rate, updates[q], sel_wss[q % ns], stream=streams[q % ns])
        if ns > 1:
            for st in streams:
                main.wait_event(st.record_event())

    def step():
        selects()
        ac.adacomp_apply(params, state, queue, lr, app_ws)

    copy_ceiling = None
    if cfg == "flat" and not args.no_copy_ceiling:     # a plain device copy: reads 4e9 bytes, writes 4e9 bytes
        src = torch.cat([g.view(-1) for g in grads[0]])
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        copy_ceiling = 5 * 2 * 4.0 * src.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    dominant = "small" if small else "filter"
    if args.graph:
        # a recorded step fixes addresses, sizes and the pulls relative to the queue: exactly what every step
        # of this bench repeats.  Replays need no host work beyond one launch.
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()
        torch.cuda.synchronize()
        t_begin = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        t_end = time.perf_counter()
        ac.adacomp_profile_start({dominant, "sweep", "bounds"})
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        prof = ac.adacomp_profile_stop()
    else:
        ac.adacomp_profile_start({dominant, "sweep", "bounds"})
        t_begin = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        t_end = time.perf_counter()
        prof = ac.adacomp_profile_stop()

    sec = t_end - t_begin
    ms_per_step = 1e3 * sec / args.steps
    value = Q * N * args.steps / sec

    f_ms, f_n = prof[dominant]
    f_avg_s = 1e-3 * f_ms / f_n
    # every element read once, every selected pair written; a step's worker gradients go through the
    # kernel in one or more launches (the library groups tensors so that a group's candidates stay cached)
    launches_per_step = f_n / args.steps
    alg_bytes = Q * (4.0 * N + 8.0 * cap) / launches_per_step
    achieved = alg_bytes / f_avg_s / 1e9
    traffic = apply_traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_flat.md")
    if os.path.exists(tpath) and cfg == "flat":   # HBM bytes per step from the committed rocprofv3 --pmc summary
        with open(tpath) as f:
            text = f.read()
        m = re.search(r"k_filter HBM bytes per step:\s*(\d+)", text)
        traffic = float(m.group(1)) / launches_per_step if m else None
        m = re.search(r"apply HBM bytes per step:\s*(\d+)", text)
        apply_traffic = float(m.group(1)) if m else None
    # the apply's kernels (slice bounds + sweep; the scatter plan has no such kernels): Sec. 4 "Complexity" counts
    # work per received entry; algorithmic bytes per entry = 40 (index 4, value 4, Theta 4R + 4W, staleness
    # bookkeeping 24), the figure the scope table states for the method, whatever plan executes it
    apply_roof = None
    if "sweep" in prof:
        a_ms = (prof["sweep"][0] + prof.get("bounds", (0.0, 0))[0]) / prof["sweep"][1]
        a_bytes = 40.0 * Q * cap
        a_ach = a_bytes / (a_ms * 1e-3) / 1e9
        apply_roof = {"bound": "hbm", "kernel": "k_bounds + sweep kernel (one launch each per queue)", "achieved": a_ach,
                      "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": a_ach / HBM_PEAK_GBS, "traffic": apply_traffic,
                      "algorithmic_bytes_per_launch": a_bytes, "avg_launch_ms": a_ms, "launches": prof["sweep"][1],
                      "bytes_per_entry": 40, "entries_per_launch": Q * cap}
    whole_bytes = Q * (4.0 * N + 8.0 * cap) + 40.0 * Q * cap
    whole = {"algorithmic_bytes_per_step": whole_bytes, "achieved_GBps": whole_bytes / (ms_per_step * 1e-3) / 1e9,
             "frac_of_peak": whole_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
             "what": "select: 4 B per element read + 8 B per selected entry written; apply: 40 B per queued entry"}
    out = {
        "metric": "gradient elements/sec compressed+applied",
        "value": value, "unit": "elements/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": ("flat: 100 tensors x 10M fp32 = 1e9 elements per worker gradient, "
                                "95% N(0,1e-5) + 5% N(0,1e-2), rate 0.5% per tensor, 16 queued updates, "
                                "staleness U[1,16]; step = select of the 16 worker gradients + 1 apply of the queue")
                   if cfg == "flat" else
                   (f"paper_cnn: 8 tensors, 211,690 fp32 parameters (Sec. 5.1), heavy-tailed gradients, rate {rate} per "
                    "tensor, 200 queued worker updates, staleness U[1,200]; step = select of the 200 worker gradients "
                    "+ 1 apply of the queue (latency regime: microseconds of work per launch)")
                   if small else
                   (f"{cfg}: {L} tensors, {N} fp32 parameters, {c['dist']} gradients, rate {rate} per tensor, {Q} queued "
                    f"worker updates, staleness U[1,{c['max_staleness']}]; step = select of the {Q} worker gradients + "
                    "1 apply of the queue"),
                   "select_calls_per_step": 1 if batched else Q, "select_streams": ns, "hip_graph": bool(args.graph),
                   "elements_per_step": Q * N, "entries_per_update": cap, "queue": Q,
                   "resident_batches": nb, "resident_gradient_bytes": 4 * nb * Q * N, "settle_s": settle_s,
                   "row_spread": args.row_spread, "rows_shared": bool(args.rows_shared)},
        "roofline": {"bound": "hbm", "kernel": "k_small" if small else "k_filter", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "algorithmic_bytes_per_launch": alg_bytes, "avg_launch_ms": 1e3 * f_avg_s,
                     "launches": f_n},
        "whole_path": whole,
    }
    if apply_roof:
        out["roofline_apply"] = apply_roof

    # split of the step between the two halves (untimed extra steps, whole-call events)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    kernels = None
    if args.breakdown:
        ac.adacomp_profile_start(None)
    ev[0].record()
    selects()
    ev[1].record()
    ac.adacomp_apply(params, state, queue, lr, app_ws)
    ev[2].record()
    torch.cuda.synchronize()
    if args.breakdown:
        kernels = {k: {"ms_total": round(v[0], 4), "launches": v[1]} for k, v in ac.adacomp_profile_stop().items()}
    sel_ms, app_ms = ev[0].elapsed_time(ev[1]) / Q, ev[1].elapsed_time(ev[2])   # select time per worker gradient
    out["select_ms_per_update"] = sel_ms
    out["apply_ms_per_queue"] = app_ms
    out["select_algorithmic_frac_of_peak"] = (4.0 * N + 8.0 * cap) / (sel_ms * 1e-3) / 1e9 / HBM_PEAK_GBS
    out["apply_entries_per_s"] = Q * cap / (app_ms * 1e-3)
    if kernels:
        out["kernels"] = kernels
    if copy_ceiling is not None:   # what a plain device copy of 4 GB reaches on this machine (read + write bytes per second)
        out["copy_ceiling_GBps"] = copy_ceiling
        out["whole_path"]["frac_of_copy_ceiling"] = out["whole_path"]["achieved_GBps"] / copy_ceiling

    if cfg == "flat" and batched and not args.no_per_gradient:
        # the same step with one adacomp_select call per worker gradient (a worker selects its own gradient):
        # the small per-call kernels are then paid 16 times
        pg_ws = torch.empty(ac.adacomp_select_workspace(sizes, rate), dtype=torch.uint8, device=dev)
        pg_updates = [ac.Update(L, cap, dev) for _ in range(Q)]
        pg_layers_of = [[ac.Layers(g) for g in bt] for bt in batches]
        for q in range(Q):
            ac.adacomp_select(pg_layers_of[0][q], rate, pg_updates[q], pg_ws)
        pg_queue = ac.Queue(pg_updates)
        pg_app_ws = torch.empty(max(256, ac.adacomp_apply_workspace(sizes, pg_updates)), dtype=torch.uint8, device=dev)

        def pg_step():
            t0 = state.t
            b = step_no[0] % nb
            step_no[0] += 1
            for q in range(Q):
                pg_updates[q].pull_ts = t0 + pulls[q]
                ac.adacomp_select(pg_layers_of[b][q], rate, pg_updates[q], pg_ws)
            ac.adacomp_apply(params, state, pg_queue, lr, pg_app_ws)

        pg_steps = max(nb, args.steps // 2 // nb * nb)
        for _ in range(2):
            pg_step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(pg_steps):
            pg_step()
        torch.cuda.synchronize()
        pg_ms = 1e3 * (time.perf_counter() - t0) / pg_steps
        out["per_gradient_calls"] = {"ms_per_step": pg_ms, "value": Q * N / (pg_ms * 1e-3), "unit": "elements/s",
                                     "steps": pg_steps, "select_calls_per_step": Q}
        del pg_ws, pg_updates, pg_layers_of, pg_queue, pg_app_ws

    if cfg == "flat" and not args.no_gpu_state:
        st_ = gpu_state(step, torch)
        if st_:
            out["gpu_state"] = st_

    if args.wire:      # one worker update (100 tensors x 50,000 entries) through the wire format and back
        u = updates[0]
        off = u.offsets
        wire = torch.empty(ac.adacomp_wire_bound(off), dtype=torch.int32, device=dev)
        nwords = torch.zeros(1, dtype=torch.int64, device=dev)
        wws = torch.empty(max(256, ac.adacomp_wire_workspace(off)), dtype=torch.uint8, device=dev)
        back = ac.Update(L, cap, dev)
        for l in range(L + 1):
            back.layer_off[l] = off[l]
        flags = torch.zeros(1, dtype=torch.int32, device=dev)
        ac.adacomp_wire_pack(u, wire, nwords, wws)
        words = int(nwords.item())
        reps = 20
        tm = []
        for fn in (lambda: ac.adacomp_wire_pack(u, wire, nwords, wws),
                   lambda: ac.adacomp_wire_unpack(wire, words, back, flags, wws)):
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            tm.append(1e3 * e0.elapsed_time(e1) / reps)
        assert int(flags.item()) == 0 and torch.equal(back.idx[:cap], u.idx[:cap]) and \
            torch.equal(back.val[:cap].view(torch.int32), u.val[:cap].view(torch.int32))
        out["wire"] = {"entries": cap, "stream_bytes": 4 * words, "bytes_per_entry": 4.0 * words / cap,
                       "raw_pairs_bytes": 8 * cap, "paper_model_bytes": 4 * cap,
                       "pack_us": tm[0], "unpack_us": tm[1],
                       "pack_GBps": (8.0 * cap + 4.0 * words) / (tm[0] * 1e-6) / 1e9,
                       "unpack_GBps": (8.0 * cap + 4.0 * words) / (tm[1] * 1e-6) / 1e9}

    if not args.no_cpu_baseline:
        del grads, batches
        out["cpu_baseline"] = cpu_baseline(cfg, rate, lr, pulls)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
