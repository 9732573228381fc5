#!/usr/bin/env python3
"""Benchmark of the Sparbit Allgather hot path on one MI355X.

One "step" is one whole Allgather call (own-block placement + all
ceil(log2 p) schedule steps) over one batch of synthetic input that is already
resident in HBM.  Prints ONE JSON line.  The headline workload is cfg4 (p=128
virtual ranks, 1 MiB blocks, 16 GiB of receive buffers): the large-block,
HBM-bound configuration the metric's bandwidth target is stated for.

  value      effective Allgather GB/s = p*p*B / t   (bytes landed per second)
  roofline   algorithmic HBM bytes (every delivered byte read once and written
             once: 2*p*p*B per call) / time, against the 8 TB/s HBM peak; time
             is taken with HIP events on the launch stream over the timed
             region
  cpu_baseline  the CPU oracle timed on this host on a bounded sample of the
             same workload (same p, smaller blocks)
  per_config other configs, context schedules and a device memcpy ceiling,
             5 warm-up + 20 timed calls each (protocol of the paper's Section
             IV-A, shortened)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak

# HBM bytes per launch of the step kernel, measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (one run each,
# scaled by a plain 1 GiB copy through the same kernel); figures and commands: profiles/copy_tiles_kernel_cfg4.md
# and profiles/copy_tiles_kernel_cfg5.md.
# Only meaningful for the default tuning and issue mode of that workload.
MEASURED_TRAFFIC_BYTES_PER_CALL = {"cfg4": (16779229 + 16777216) * 1024, "cfg5": (16916835 + 16908544) * 1024}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg4",
                    help="cfg1 .. cfg5, or pP_bB for P ranks with blocks of B bytes (uint8 payload), e.g. p128_b1048580")
    ap.add_argument("--mode", default="auto", choices=["auto", "per_step", "persistent", "dataflow"])
    ap.add_argument("--skip-context", action="store_true", help="only the headline workload")
    ap.add_argument("--skip-cpu-baseline", action="store_true")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE")
    ap.add_argument("--sweep", metavar="OUT.jsonl", default=None,
                    help="instead of the benchmark: time every schedule over the block-size ladder 1 B .. 1 MiB "
                         "(doubling, as OSU's osu_allgather in the paper's Section IV-A) for process counts on the "
                         "paper's two progressions, one JSON line per case into OUT.jsonl")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="instead of the benchmark: --steps plain 1 GiB copies (p=1 own-block placement), "
                         "the known-size kernel that scales the rocprofv3 HBM counters")
    return ap.parse_args()


def time_calls(torch, fn, stream, warmup, steps):
    """Average / min / max milliseconds per call; events sit on `stream`."""
    with torch.cuda.stream(stream):
        for _ in range(warmup):
            fn()
        stream.synchronize()
        torch.cuda.synchronize()
        t_wall = time.perf_counter()
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        evs[0].record(stream)
        for i in range(steps):
            fn()
            evs[i + 1].record(stream)
        stream.synchronize()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t_wall) * 1e3
    per = [evs[i].elapsed_time(evs[i + 1]) for i in range(steps)]
    total = evs[0].elapsed_time(evs[steps])
    return {"avg_ms": total / steps, "min_ms": min(per), "max_ms": max(per), "wall_ms_per_call": wall_ms / steps}


def make_device_send(torch, w, dev):
    from paper_2109_08751_amd import workloads
    return torch.from_numpy(workloads.make_send(w)).to(dev)


def rates(p, B, ms):
    landed = p * p * B
    return {"effective_GBps": landed / ms / 1e6, "hbm_GBps": 2 * landed / ms / 1e6,
            "hbm_frac": 2 * landed / ms / 1e6 / HBM_PEAK_GBPS}


def cpu_baseline(w):
    """Time the oracle (single-threaded C simulation) on the same p with smaller
    blocks, sized from a short probe so that it costs roughly 10 s."""
    import numpy as np
    import oracle
    from paper_2109_08751_amd import workloads

    p = w.p

    def run(B):
        send = np.tile(workloads.make_send_raw(p, min(B, 4096), 1), (1, max(B // 4096, 1)))[:, :B].copy()
        recv = np.full((p, p, B), workloads.POISON, dtype=np.uint8)
        t = time.perf_counter()
        oracle.allgather(oracle.SPARBIT, p, B, send, recv)
        dt = time.perf_counter() - t
        assert (recv[p - 1, 0] == send[0]).all()
        return dt

    B = max(16, min(w.block_bytes, 4096))
    dt = run(B)
    rate = p * p * B / dt
    target = max(B, min(w.block_bytes, int(rate * 10.0 / (p * p))))
    Bs = 1 << (target.bit_length() - 1)
    avail = 0
    try:
        for line in open("/proc/meminfo"):
            if line.startswith("MemAvailable:"):
                avail = int(line.split()[1]) * 1024
    except OSError:
        pass
    # the oracle holds the receive buffers plus a mailbox of up to half their size
    while Bs > B and 2 * p * p * Bs > max(avail // 2, 1 << 30):
        Bs >>= 1
    if Bs > B:
        dt, B = run(Bs), Bs
    model, mem_total = "unknown", 0
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
        for line in open("/proc/meminfo"):
            if line.startswith("MemTotal:"):
                mem_total = int(line.split()[1]) * 1024
    except OSError:
        pass
    return {"value": p * p * B / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "seconds": dt,
            "host": {"cpu_model": model, "nproc": os.cpu_count(), "mem_total_GiB": round(mem_total / 2**30, 1)},
            "sample": f"Sparbit oracle, p={p}, block {B} B (workload block {w.block_bytes} B), "
                      f"recv {p * p * B / 2**20:.0f} MiB, one pass"}


def sweep(torch, sb, workloads, stream, path):
    """Latency/bandwidth ladder in the shape of the paper's test matrix (Section IV-A): block sizes 1 B .. 1 MiB by
    doubling; p from the even/power-of-two progression (8, 16, ..., 256) and the odd one (5, 13, ..., 253), thinned."""
    dev = torch.device("cuda:0")
    ps = [8, 16, 32, 64, 128, 256, 5, 13, 29, 61, 125, 253]
    sizes = [1 << k for k in range(0, 21)]
    algos = [("sparbit", sb.SPARBIT), ("ring", sb.RING), ("recursive_doubling", sb.RECURSIVE_DOUBLING),
             ("bruck", sb.BRUCK), ("direct", sb.DIRECT)]
    n = 0
    with open(path, "w") as out:
        for p in ps:
            for B in sizes:
                if p * p * B > (32 << 30):
                    continue
                send = torch.randint(0, 256, (p, B), dtype=torch.uint8, device=dev)
                recv = torch.full((p, p, B), workloads.POISON, dtype=torch.uint8, device=dev)
                for label, algo in algos:
                    if algo == sb.RECURSIVE_DOUBLING and p & (p - 1):
                        continue
                    if algo == sb.RING and p * p * B > (1 << 30):
                        continue  # p - 1 launches of tiny kernels each: skipped where it only burns time
                    fn = lambda: sb.sparbit_allgather_mode(send, recv, p, B, algo, sb.MODE_AUTO, stream)
                    t = time_calls(torch, fn, stream, 3, 10)
                    ok = bool(torch.equal(recv, send.unsqueeze(0).expand(p, p, B))) if p * p * B <= (1 << 28) \
                        else bool(torch.equal(recv[p - 1], send))
                    out.write(json.dumps({"p": p, "block_bytes": B, "algo": label, "ok": ok,
                                          "avg_us": t["avg_ms"] * 1e3, "min_us": t["min_ms"] * 1e3,
                                          "max_us": t["max_ms"] * 1e3,
                                          "effective_GBps": p * p * B / t["avg_ms"] / 1e6}) + "\n")
                    out.flush()
                    n += 1
                    recv.fill_(workloads.POISON)
                del send, recv
            print(f"sweep: p={p} done ({n} cases)", file=sys.stderr, flush=True)
            torch.cuda.empty_cache()
    return n


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (all virtual ranks share one HBM); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    import paper_2109_08751_amd as sb
    from paper_2109_08751_amd import workloads

    for kv in args.tune:
        k, v = kv.split("=")
        sb.sparbit_tune(k, int(v))
    mode = {"auto": sb.MODE_AUTO, "per_step": sb.MODE_PER_STEP, "persistent": sb.MODE_PERSISTENT,
            "dataflow": sb.MODE_DATAFLOW}[args.mode]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.Stream()
    if args.sweep:
        n = sweep(torch, sb, workloads, stream, args.sweep)
        assert sb.sparbit_barrier_timeouts(stream) == 0
        print(json.dumps({"sweep_cases": n, "file": args.sweep}))
        return
    if args.calibrate_copy:
        nbytes = 1 << 30
        src = torch.full((nbytes,), 7, dtype=torch.uint8, device=dev)
        dst = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
        t = time_calls(torch, lambda: sb.sparbit_allgather_mode(src, dst, 1, nbytes, sb.SPARBIT, sb.MODE_PER_STEP, stream),
                       stream, args.warmup, args.steps)
        print(json.dumps({"calibrate_copy_bytes_each_way": nbytes, "launches": args.warmup + args.steps,
                          "ok": bool(torch.equal(src, dst)), **t, **rates(1, nbytes, t["avg_ms"])}))
        return
    if args.workload in workloads.WORKLOADS:
        w = workloads.WORKLOADS[args.workload]
    else:
        import re
        m = re.fullmatch(r"p(\d+)_b(\d+)", args.workload)
        if not m:
            print(f"bench.py: unknown workload {args.workload!r}", file=sys.stderr)
            sys.exit(2)
        w = workloads.Workload(args.workload, int(m.group(1)), int(m.group(2)), "u8",
                               f"p={m.group(1)}, {m.group(2)}-byte uint8 blocks")
    p, B = w.p, w.block_bytes

    # ---- headline: timed region of exactly --steps calls
    d_send = make_device_send(torch, w, dev)
    d_recv = torch.full((p, p, B), workloads.POISON, dtype=torch.uint8, device=dev)
    call = lambda: sb.sparbit_allgather_mode(d_send, d_recv, p, B, sb.SPARBIT, mode, stream)
    head = time_calls(torch, call, stream, args.warmup, args.steps)
    assert sb.sparbit_barrier_timeouts(stream) == 0
    ok = all(bool(torch.equal(d_recv[r], d_send)) for r in (0, p // 2, p - 1))
    if not ok:
        print("bench.py: result check failed", file=sys.stderr)
        sys.exit(1)
    r = rates(p, B, head["avg_ms"])
    nsteps = sb.Plan(p).num_steps
    launches = 1 if mode in (sb.MODE_PERSISTENT, sb.MODE_DATAFLOW) else nsteps  # own blocks + step 0 share the first launch
    out = {
        "metric": "effective Allgather GB/s (p*p*block_bytes landed / time; % of MI355X peak HBM BW in "
                  "roofline.frac), Sparbit schedule, per p and block size",
        "value": r["effective_GBps"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["avg_ms"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.note}; recv {w.recv_bytes / 2**30:.2f} GiB; {nsteps} steps",
                   "p": p, "block_bytes": B, "mode": args.mode},
        "min_ms": head["min_ms"], "max_ms": head["max_ms"], "wall_ms_per_step": head["wall_ms_per_call"],
        "schedule_only_GBps": p * (p - 1) * B / head["avg_ms"] / 1e6,  # without the own-block placement
        "roofline": {"bound": "hbm", "achieved": r["hbm_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": r["hbm_frac"],
                     "traffic": (MEASURED_TRAFFIC_BYTES_PER_CALL[w.name] / launches
                                 if w.name in MEASURED_TRAFFIC_BYTES_PER_CALL and not args.tune and args.mode == "auto"
                                 else None),
                     "kernel": ("sparbit::copy_tiles_kernel<unsigned int __vector(4), unsigned int, %d, 1, true, false, true>"
                                % (64 if 8192 <= B <= (4 << 20) else 256)
                                if B % 16 == 0 else "sparbit::copy_tiles_realign_kernel<256, true>"),
                     "launches_per_call": launches,
                     "algorithmic_bytes_per_launch": 2 * p * p * B / launches,
                     "avg_launch_ms": head["avg_ms"] / launches,
                     "note": "achieved = algorithmic bytes per launch (2*p*p*B / launches) / average launch "
                             "duration, the latter from HIP events on the launch stream over the timed region "
                             "(launch gaps included); traffic = measured HBM bytes per launch"},
    }
    del d_recv

    # ---- context: other configs, other schedules, memcpy ceiling
    if not args.skip_context:
        per = {}
        for name in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5"):
            wc = workloads.WORKLOADS[name]
            pc, Bc = wc.p, wc.block_bytes
            s_ = d_send if name == w.name else make_device_send(torch, wc, dev)
            r_ = torch.full((pc, pc, Bc), workloads.POISON, dtype=torch.uint8, device=dev)
            row = {"p": pc, "block_bytes": Bc}
            algos = [("sparbit", sb.SPARBIT, sb.MODE_AUTO), ("direct", sb.DIRECT, sb.MODE_AUTO)]
            if name in ("cfg1", "cfg2", "cfg3"):
                algos += [("sparbit_dataflow", sb.SPARBIT, sb.MODE_DATAFLOW)]
            if name in ("cfg2", "cfg3", "cfg4", "cfg5"):
                algos += [("bruck", sb.BRUCK, sb.MODE_AUTO)]
                if pc & (pc - 1) == 0:
                    algos += [("recursive_doubling", sb.RECURSIVE_DOUBLING, sb.MODE_AUTO)]
            if name in ("cfg1", "cfg2", "cfg3"):
                algos += [("ring", sb.RING, sb.MODE_AUTO)]
            for label, algo, md in algos:
                fn = lambda a=algo, m=md: sb.sparbit_allgather_mode(s_, r_, pc, Bc, a, m, stream)
                t = time_calls(torch, fn, stream, 5, 20)
                row[label] = {**t, **rates(pc, Bc, t["avg_ms"])}
                good = bool(torch.equal(r_[pc - 1], s_))
                row[label]["ok"] = good
                r_.fill_(workloads.POISON)
            # ceiling: one device-to-device memcpy of the same p*p*B bytes
            dst = torch.empty_like(r_)
            t = time_calls(torch, lambda: dst.copy_(r_, non_blocking=True), stream, 3, 10)
            row["memcpy_d2d"] = {**t, **rates(pc, Bc, t["avg_ms"])}
            per[name] = row
            del r_, dst, s_
            torch.cuda.empty_cache()
        # Allgatherv on a cfg4-shaped job: 128 ranks, block sizes spread over 0.5 .. 1.5 MiB (mean 1 MiB), at three
        # granularities: 4 KiB (every block on the 16-byte grid), 4 bytes and 1 byte (the realigning kernel).
        import numpy as np
        pv = 128
        for label, grain in (("allgatherv_p128_0.5-1.5MiB", 4096), ("allgatherv_p128_0.5-1.5MiB_grain4B", 4),
                             ("allgatherv_p128_0.5-1.5MiB_grain1B", 1)):
            rng = np.random.default_rng(workloads.DEFAULT_SEED)
            counts = (rng.integers(512 << 10, (1536 << 10) + 1, pv) // grain * grain).astype(np.uint64)
            displs = np.concatenate([[0], np.cumsum(counts[:-1])]).astype(np.uint64)
            row = int(counts.sum())
            s_ = torch.randint(0, 256, (row,), dtype=torch.uint8, device=dev)
            r_ = torch.full((pv, row), workloads.POISON, dtype=torch.uint8, device=dev)
            t = time_calls(torch, lambda: sb.sparbit_allgatherv(s_, r_, pv, counts, displs, row, sb.SPARBIT, stream),
                           stream, 3, 10)
            per[label] = {
                "p": pv, "row_bytes": row, **t, "effective_GBps": pv * row / t["avg_ms"] / 1e6,
                "hbm_GBps": 2 * pv * row / t["avg_ms"] / 1e6,
                "hbm_frac": 2 * pv * row / t["avg_ms"] / 1e6 / HBM_PEAK_GBPS,
                "ok": bool(torch.equal(r_[pv - 1], s_))}
            del s_, r_
            torch.cuda.empty_cache()
        # Equal blocks off the 16-byte grid: cfg4's shape with 4 more bytes per block
        pu, Bu = 128, (1 << 20) + 4
        s_ = torch.randint(0, 256, (pu, Bu), dtype=torch.uint8, device=dev)
        r_ = torch.full((pu, pu, Bu), workloads.POISON, dtype=torch.uint8, device=dev)
        t = time_calls(torch, lambda: sb.sparbit_allgather_mode(s_, r_, pu, Bu, sb.SPARBIT, sb.MODE_AUTO, stream),
                       stream, 3, 10)
        per["sparbit_p128_1MiB+4B"] = {"p": pu, "block_bytes": Bu, **t, **rates(pu, Bu, t["avg_ms"]),
                                       "ok": bool(torch.equal(r_[pu - 1], s_))}
        del s_, r_
        torch.cuda.empty_cache()
        out["per_config"] = per
        assert sb.sparbit_barrier_timeouts(stream) == 0

    if not args.skip_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    # Context only (Sections IV and V of the paper): another machine, another metric -- not a target.
    out["paper_context"] = {
        "hardware": "Open MPI 4.0.3, OSU osu_allgather 5.7; Yahoo: 16 nodes of 2x Xeon L5420, GbE leaves + 10 Gb/s "
                    "core; Cervino: 5 nodes of 2x Xeon E5-2683 v4, 40 Gb/s flat; 1 B..1 MiB blocks, up to 256 / 320 "
                    "processes",
        "reported": "no absolute rates; Sparbit has the best average time in 46.43 % (Yahoo) / 39.64 % (Cervino) of "
                    "the cases under sequential mapping, improving on the second best by 34.70 / 26.16 / 84.16 % "
                    "(mean / median / highest, Yahoo) and 30.23 / 29.00 / 77.78 % (Cervino)"}
    sb.sparbit_finalize()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
