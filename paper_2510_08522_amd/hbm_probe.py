"""What the memory system of the device gives a kernel shaped like the streaming pass.

Runs the plain streaming kernels behind dynamix_hbm_probe (no arithmetic; one block of 256
threads per compute unit, contiguous span per block, 128-bit non-temporal accesses) and prints,
as text and as one JSON line, the rates against which the streaming pass is judged:

  read-only     K buffers of P fp32 elements, consecutive 4 KB tiles and interleaved chunks
  write-only    P fp32 elements
  copy          one buffer to another (at most 1 GiB)
  read | write  the read-only kernel on (units - n) compute units while a write-only kernel on
                the other n units writes P fp32 elements once, on a second stream: how much a
                byte written costs the read stream when both are in the memory system

Run as `python -m paper_2510_08522_amd.hbm_probe` (defaults: the K = 32, P = 138 M shape).
"""
import argparse
import json
import sys

import torch

from . import binding as B


def _time(fn, reps, stream=None):
    """Average milliseconds of fn() over reps launches on the current stream, after two warm-ups."""
    for _ in range(2):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--streams", type=int, default=32, choices=[1, 2, 4, 8, 16, 32])
    ap.add_argument("--elements", type=int, default=138_000_000, help="fp32 elements per buffer")
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--settle-seconds", type=float, default=2.0)
    args = ap.parse_args(argv)
    if not torch.cuda.is_available():
        sys.exit("hbm_probe: no GPU visible")
    B.load()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(0)
    units = torch.cuda.get_device_properties(0).multi_processor_count
    K, P = args.streams, args.elements
    nbytes = P * 4 // 4096 * 4096
    bufs = [torch.empty(P, dtype=torch.float32, device=dev).normal_() for _ in range(K)]
    dst = torch.empty(P, dtype=torch.float32, device=dev)
    res = {"units": units, "streams": K, "bytes_per_buffer": nbytes}
    out = []

    def say(s):
        print(s, flush=True)
        out.append(s)

    # settle the clocks
    import time
    t_end = time.perf_counter() + args.settle_seconds
    while time.perf_counter() < t_end:
        B.dynamix_hbm_probe(bufs, nbytes, B.DYNAMIX_PROBE_READ_SPREAD, units)
        torch.cuda.synchronize()

    for name, mode in (("read_consecutive", B.DYNAMIX_PROBE_READ),
                       ("read_interleaved", B.DYNAMIX_PROBE_READ_SPREAD),
                       ("read_interl_128B", B.DYNAMIX_PROBE_READ_SPREAD_128B),
                       ("read_interl_512B", B.DYNAMIX_PROBE_READ_SPREAD_512B)):
        ms = _time(lambda: B.dynamix_hbm_probe(bufs, nbytes, mode, units), args.reps)
        res[name] = {"ms": ms, "GBps": K * nbytes / ms / 1e6}
        say("%-18s %d x %.1f MB: %.4f ms  %.0f GB/s" % (name, K, nbytes / 1e6, ms, K * nbytes / ms / 1e6))
    ms = _time(lambda: B.dynamix_hbm_probe([dst], nbytes, B.DYNAMIX_PROBE_WRITE, units), args.reps)
    res["write_only"] = {"ms": ms, "GBps": nbytes / ms / 1e6}
    say("%-18s %.1f MB: %.4f ms  %.0f GB/s" % ("write_only", nbytes / 1e6, ms, nbytes / ms / 1e6))
    cb = min(nbytes, 1 << 30)
    ms = _time(lambda: B.dynamix_hbm_probe([bufs[0], dst], cb, B.DYNAMIX_PROBE_COPY, units), args.reps)
    res["copy"] = {"ms": ms, "GBps_read_plus_write": 2 * cb / ms / 1e6}
    say("%-18s %.1f MB: %.4f ms  %.0f GB/s read + written" % ("copy", cb / 1e6, ms, 2 * cb / ms / 1e6))

    # reading while another kernel writes, on disjoint compute units, two streams
    s_r, s_w = torch.cuda.Stream(), torch.cuda.Stream()
    res["read_beside_write"] = []
    for n in (0, 8, 16, 32, 64):
        t_r, t_w = [], []
        for rep in range(2 + args.reps // 2):
            er0, er1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ew0, ew1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            with torch.cuda.stream(s_r):
                er0.record()
                B.dynamix_hbm_probe(bufs, nbytes, B.DYNAMIX_PROBE_READ_SPREAD, units - n, stream=s_r)
                er1.record()
            if n:
                with torch.cuda.stream(s_w):
                    ew0.record()
                    B.dynamix_hbm_probe([dst], nbytes, B.DYNAMIX_PROBE_WRITE, n, stream=s_w)
                    ew1.record()
            torch.cuda.synchronize()
            if rep >= 2:
                t_r.append(er0.elapsed_time(er1))
                if n:
                    t_w.append(ew0.elapsed_time(ew1))
        r = sum(t_r) / len(t_r)
        w = sum(t_w) / len(t_w) if t_w else 0.0
        res["read_beside_write"].append({"write_units": n, "read_ms": r, "write_ms": w})
        say("read on %3d units: %.4f ms%s" % (
            units - n, r,
            "" if not n else "   write of %.0f MB on %2d units beside it: %.4f ms (%.0f GB/s)"
            % (nbytes / 1e6, n, w, nbytes / w / 1e6)))
    print(json.dumps(res), flush=True)
    return res


if __name__ == "__main__":
    main()
