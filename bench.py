"""Throughput of the gradient aggregate + statistics hot path on one MI355X.

A step is one call of dynamix_grad_aggregate_stats_ex (streaming pass + final reduction) over the
K gradient buffers of one synthetic workload, all resident in HBM before the timed region.
Prints one JSON line: gradient GB/s processed (K*P*sizeof(dtype) per step), the roofline figures
of the dominant kernel measured with HIP events recorded around it on its own stream, and the
CPU oracle timed on a bounded sample of the same inputs on the host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak

# HBM bytes per launch of the streaming pass from rocprofv3 counters (FETCH_SIZE + WRITE_SIZE,
# each scaled by the reading of a plain copy of known size), keyed by workload, and the hash of
# the kernel source they were taken on.  A changed kernel makes the figure stale: traffic = null.
MEASURED_TRAFFIC = {"C4": {"bytes": 18218544120, "kernel": "9a0ba85c62a2bcc9"},
                    "C3": {"bytes": 922842482, "kernel": "9a0ba85c62a2bcc9"},
                    "C5": {"bytes": 4466021018, "kernel": "9a0ba85c62a2bcc9"}}
KERNEL_FILES = ("stream_pass.h", "dynamix_internal.h", "stream_pass_inst.hip")


def kernel_source_hash():
    import hashlib
    h = hashlib.sha256()
    for f in KERNEL_FILES:
        with open(os.path.join(ROOT, "paper_2510_08522_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def describe(w):
    seg = "single segment" if w.S == 0 else "%d segments" % w.S
    dt = "bf16" if w.itemsize == 2 else "fp32"
    return "%s: K=%d workers, P=%d %s gradients, %s" % (w.name, w.K, w.P, dt, seg)


def cpu_model():
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(w, sample_elems, threads):
    """Times the CPU oracle, as it stands, on the first `sample_elems` elements of every worker
    buffer (copied to the host outside the timed part)."""
    import oracle
    n = min(sample_elems, w.P)
    off = None
    if w.segment_offsets is not None:
        off = [int(o) for o in w.segment_offsets if o < n] + [n]
    host = w.host_arrays(0, n)
    threads = max(1, min(threads, oracle.max_threads()))
    t0 = time.perf_counter()
    oracle.aggregate_stats(host, w.batch_sizes, off, want_agg=True, threads=threads)
    dt = time.perf_counter() - t0
    nbytes = w.K * n * w.itemsize
    # the same oracle on one thread, on a sixteenth of that sample
    n1 = max(1, n // 16)
    off1 = None if off is None else [o for o in off if o < n1] + [n1]
    host1 = [h[:n1] for h in host]
    t0 = time.perf_counter()
    oracle.aggregate_stats(host1, w.batch_sizes, off1, want_agg=True, threads=1)
    dt1 = time.perf_counter() - t0
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
            "nproc": os.cpu_count(), "cpu_model": cpu_model(),
            "sample": "first %d of %d elements of each of the %d worker buffers "
                      "(%.3f GB read, %.2f s wall)" % (n, w.P, w.K, nbytes / 1e9, dt),
            "elements_per_s": w.K * n / dt,
            "single_thread": {"value": w.K * n1 * w.itemsize / dt1 / 1e9, "unit": "GB/s",
                              "sample": "first %d elements of each buffer, %.2f s wall"
                                        % (n1, dt1)}}


def memory_ceiling(D, torch, sets, w, stream):
    """What the memory system gives plain streaming kernels of the streaming pass's launch shape on
    this workload's own buffers, measured after the timed region (dynamix_hbm_probe: no
    arithmetic): the K buffers read and nothing written, the aggregate's bytes written and nothing
    read.  Their sum is the time of a pass that lost nothing where reads and writes meet."""
    B = D.binding
    if w.K not in (1, 2, 4, 8, 16, 32):
        return None
    if any(g.data_ptr() % 256 for s in sets for g in s[0]) or any(s[1].data_ptr() % 256 for s in sets):
        return None
    units = torch.cuda.get_device_properties(0).multi_processor_count
    if w.P * w.itemsize < 64 * 4096 * units:     # under 64 tiles per block the probe is not at speed
        return None
    in_bytes = w.P * w.itemsize // 4096 * 4096
    out_bytes = w.P * 4 // 4096 * 4096
    reps = max(10, min(200, int(2e10 // max(w.bytes_read, 1))))
    n = [0]

    def timed(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    def read():
        grads = sets[n[0] % len(sets)][0]
        n[0] += 1
        B.dynamix_hbm_probe(grads, in_bytes, B.DYNAMIX_PROBE_READ_SPREAD, units, stream=stream)

    def write():
        agg = sets[n[0] % len(sets)][1]
        n[0] += 1
        B.dynamix_hbm_probe([agg], out_bytes, B.DYNAMIX_PROBE_WRITE, units, stream=stream)

    r_ms, w_ms = timed(read), timed(write)
    return {"read_only_ms": round(r_ms, 5), "read_only_GBps": round(w.K * in_bytes / r_ms / 1e6, 1),
            "write_only_ms": round(w_ms, 5), "write_only_GBps": round(out_bytes / w_ms / 1e6, 1),
            "read_then_write_ms": round(r_ms + w_ms, 5),
            "read_then_write_GBps_of_read_bytes": round(w.bytes_read / (r_ms + w_ms) / 1e6, 1),
            "note": "plain streaming kernels (no arithmetic) on the same buffers; the last two "
                    "figures assume no cost where reads and writes meet"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C4", choices=["C1", "C2", "C3", "C4", "C5", "wide"],
                    help="one of the five named configurations, or 'wide': --workers (more than 64: "
                         "the two-sweep kernel) fp32 buffers of --elements, C4's generator")
    ap.add_argument("--workers", type=int, default=128)
    ap.add_argument("--elements", type=int, default=34_500_000)
    ap.add_argument("--update", default="none", choices=["none", "sgd", "momentum", "adam"],
                    help="time the pass with this model update fused in instead of the write of the "
                         "aggregate (momentum, adam: up to 32 workers)")
    ap.add_argument("--cpu-sample", type=int, default=16_000_000,
                    help="elements per worker the CPU oracle is timed on (0: skip)")
    ap.add_argument("--cpu-threads", type=int, default=16)
    ap.add_argument("--one-allocation", action="store_true",
                    help="make the K gradient buffers rows of one allocation instead of K "
                         "allocations made one by one")
    ap.add_argument("--settle-seconds", type=float, default=2.0,
                    help="run the step untimed for this long before the warm-up steps: right after "
                         "other heavy GPU work the device takes a second or two to reach its steady "
                         "clocks (kernel time 3-4 %% longer until then)")
    ap.add_argument("--warm", action="store_true",
                    help="time one input set over and over even when it fits the 256 MB "
                         "memory-side cache (default: rotate copies of it so every step reads "
                         "from HBM)")
    ap.add_argument("--stagger-elems", type=int, default=0,
                    help="without --one-allocation: start buffer k that many elements times k "
                         "into its allocation (a multiple of 8), so that the K streams do not sit "
                         "at the same offsets of their allocations")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain elementwise copy of 2^28 floats (1 GiB read, 1 GiB "
                         "written) three times, as the known-size reference for HBM byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this path runs on one GPU only (no sharding, no collectives); "
                 "run with --gpus 1")

    import torch
    import paper_2510_08522_amd as D
    from paper_2510_08522_amd import workloads as W

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    if not os.path.exists(D.binding.LIB_PATH):   # load what is built; build only if nothing is
        from paper_2510_08522_amd import build as _build
        _build.build()
    D.binding.load()                      # no fallback: raises if the library cannot be loaded
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.workload == "wide":
        import numpy as np
        seed = W.BASE_SEED + 6
        b = np.random.default_rng(seed).integers(16, 257, size=args.workers)
        w = W.make(args.workers, args.elements, torch.float32, b, 1e-3, 1e-2, seed, device=dev,
                   name="wide", one_allocation=args.one_allocation)
    else:
        w = W.config(args.workload, device=dev, one_allocation=args.one_allocation,
                     stagger_elems=0 if args.one_allocation else args.stagger_elems)
    # streams the pass writes per element (and, but for the plain aggregate, reads first)
    n_state = {"none": 0, "sgd": 1, "momentum": 2, "adam": 3}[args.update]
    out_agg = torch.zeros(w.P, dtype=torch.float32, device=dev)
    out_stats = torch.empty((1 + w.S, D.DYNAMIX_STATS_HEAD + 2 * w.K), dtype=torch.float64,
                            device=dev)
    stream = torch.cuda.current_stream()

    # Cold-cache protocol: a workload that the 256 MB memory-side cache could hold between steps
    # is timed on a rotation of copies at distinct addresses, together more than twice the cache.
    CACHE = 256 << 20
    state = [torch.zeros(w.P, dtype=torch.float32, device=dev) for _ in range(max(0, n_state - 1))]
    sets = [(w.grads, out_agg)]
    if w.bytes_read + w.P * 4 > 2 * CACHE:
        cache_note = "cold by size: one step streams %.0f MB through a 256 MB cache" % (
            (w.bytes_read + w.P * 4) / 1e6)
    elif args.warm:
        cache_note = "warm: the same %.0f MB every step" % (w.bytes_read / 1e6)
    else:
        copies = -(-(5 * CACHE // 2) // (w.bytes_read + w.P * 4))
        for _ in range(copies - 1):
            sets.append(([g.clone() for g in w.grads], torch.zeros_like(out_agg)))
        cache_note = "cold: rotation of %d copies of the inputs at distinct addresses (%.0f MB)" % (
            copies, copies * (w.bytes_read + w.P * 4) / 1e6)
    calls = [0]

    def step():
        # (with a fused update the set's output buffer serves as the parameter vector)
        grads, agg = sets[calls[0] % len(sets)]
        calls[0] += 1
        if args.update == "none":
            D.dynamix_grad_aggregate_stats_ex(grads, w.batch_sizes, w.segment_offsets,
                                              out_agg=agg, out_stats=out_stats, stream=stream)
        elif args.update == "sgd":
            D.dynamix_grad_aggregate_stats_sgd(grads, w.batch_sizes, agg, 0.01, 1e-4,
                                               w.segment_offsets, out_stats=out_stats, stream=stream)
        elif args.update == "momentum":
            D.dynamix_grad_aggregate_stats_sgd_momentum(grads, w.batch_sizes, agg, state[0], 0.01, 1e-4,
                                                        0.9, False, w.segment_offsets,
                                                        out_stats=out_stats, stream=stream)
        else:
            D.dynamix_grad_aggregate_stats_adam(grads, w.batch_sizes, agg, state[0], state[1], 1e-3,
                                                calls[0], segment_offsets=w.segment_offsets,
                                                out_stats=out_stats, stream=stream)

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 0.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    t_end = time.perf_counter() + max(0.0, args.settle_seconds)
    while time.perf_counter() < t_end:
        for _ in range(10):
            step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # Kernel durations are sampled with HIP events on every fifth step of the timed region: the
    # three events of a timed call hold the stream up for about ten microseconds.
    every = 5 if args.steps >= 10 else 1
    D.dynamix_timing_every(every)
    D.dynamix_timing_begin(-(-args.steps // every))    # event slots are created outside the timed region
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    enqueued = time.perf_counter() - t0   # host side of the calls: marshalling, plan lookup, launches
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    n = D.dynamix_timing_count()
    times = [D.dynamix_timing_read(i) for i in range(n)]

    # the same workload without the write of the aggregate (out_agg = NULL), outside the timed
    # region: how much of the step the 4 bytes written per element cost
    so_steps = min(args.steps, 20)
    D.dynamix_timing_every(1)
    D.dynamix_timing_begin(so_steps)
    for _ in range(so_steps):
        D.dynamix_grad_aggregate_stats_ex(sets[calls[0] % len(sets)][0], w.batch_sizes,
                                          w.segment_offsets, out_stats=out_stats, stream=stream,
                                          stats_only=True)
        calls[0] += 1
    torch.cuda.synchronize()
    so_ms = sum(D.dynamix_timing_read(i)[0] for i in range(so_steps)) / so_steps
    D.dynamix_timing_begin(0)
    k_stream = sum(t[0] for t in times) / n * 1e-3      # seconds per launch
    k_final = sum(t[1] for t in times) / n * 1e-3

    ms_per_step = elapsed / args.steps * 1e3
    read_bytes = w.bytes_read
    sweeps = 2 if w.K > D.DYNAMIX_K_MAX_ONE_SWEEP else 1 # above 64 workers the gradients are read twice
    # K*s read + 4 written per element; a fused update reads and writes 4 per element and stream
    algo_bytes = sweeps * read_bytes + w.P * 4 * (1 if n_state == 0 else 2 * n_state)
    value = read_bytes / (elapsed / args.steps) / 1e9
    achieved = algo_bytes / k_stream / 1e9
    ns = float(out_stats[0, D.STAT["noise_scale"]].item())

    m = MEASURED_TRAFFIC.get(w.name) if args.update == "none" else None
    traffic = m["bytes"] if m and m["kernel"] == kernel_source_hash() else None

    line = {
        "metric": "gradient GB/s processed (aggregate+stats) and % of MI355X HBM peak",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",      # accumulation type; bf16 inputs are widened exactly
        "data": "synthetic",
        "config": {"workload": describe(w) + ("" if args.update == "none" else
                                              ", fused %s update" % args.update),
                   "K": w.K, "P": w.P, "segments": w.S, "update": args.update,
                   "input_dtype": "bf16" if w.itemsize == 2 else "fp32",
                   "bytes_read_per_step": read_bytes, "seed": w.seed,
                   "buffers": ("K allocations" + (", staggered by %d elements" % args.stagger_elems
                                                 if args.stagger_elems else ""))
                   if not args.one_allocation else "K rows of one allocation",
                   "cache": cache_note},
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "elements_per_s": w.K * w.P / (elapsed / args.steps),
        "total_traffic_GBps": round(algo_bytes / (elapsed / args.steps) / 1e9, 2),
        "noise_scale": ns,
        "host_enqueue_us_per_step": round(enqueued / args.steps * 1e6, 2),
        "settle_seconds": args.settle_seconds,
        "roofline": {"bound": "hbm", "kernel": "wide_pass_kernel" if sweeps == 2 else "stream_pass_kernel",
                     "achieved": round(achieved, 2), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "algorithmic_bytes_per_launch": algo_bytes,
                     "kernel_ms": round(k_stream * 1e3, 5), "launches_timed": n,
                     "timing": "HIP events around the kernel on its stream, every %s step of the "
                               "timed region" % ("5th" if every == 5 else "single"),
                     "final_reduce_ms": round(k_final * 1e3, 5)},
    }
    line["stats_only"] = {"kernel_ms": round(so_ms, 5),
                          "read_GBps": round(read_bytes / so_ms / 1e6, 2),
                          "frac_of_peak": round(read_bytes / so_ms / 1e6 / HBM_PEAK_GBPS, 4)}
    ceiling = memory_ceiling(D, torch, sets, w, stream) if args.update == "none" else None
    if ceiling:
        line["memory_ceiling"] = ceiling
    if args.cpu_sample > 0:
        line["cpu_baseline"] = cpu_baseline(w, args.cpu_sample, args.cpu_threads)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
