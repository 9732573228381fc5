#!/usr/bin/env python3
"""Benchmark of the Sparbit Allgather hot path on one MI355X.

One "step" is one whole Allgather call (own-block placement and every message
of the Sparbit schedule) over one batch of synthetic input that is already
resident in HBM.  Prints ONE JSON line.  The headline workload is cfg5 (p=257
virtual ranks, 256 KiB blocks, 16.13 GiB of receive buffers), the largest of
the five configurations; cfg4 and the others are rows of `per_config`.

  value      effective Allgather GB/s = p*p*B / t   (bytes landed per second)
  roofline   algorithmic HBM bytes of the dominant kernel's launches / their
             duration, against the 8 TB/s HBM peak.  The bytes depend on the
             form the library chose (it reports the kernel it launched):
               one launch per step   every delivered byte is read from HBM and
                                     written to HBM: 2*p*p*B per call
               tree kernel           a wavefront forwards what it wrote itself
                                     moments before; only the send buffer has
                                     to come from HBM: p*B + p*p*B per call
             time is taken with HIP events on the launch stream over the timed
             region
  cpu_baseline  the CPU oracle timed on this host, before the GPU is touched:
             one thread, and one unchanged single-threaded simulation per core
             on disjoint problems (the simulation itself is serial)
  per_config every configuration, the other schedules, copy ceilings through
             the library's own kernels and through the runtime's memcpy; 5
             warm-up + 20 timed calls each (protocol of the paper's Section
             IV-A, shortened)

Other uses (each instead of the benchmark):
  --sweep OUT.jsonl           the block-size ladder of Section IV-A
  --sweep-summary IN.jsonl    markdown tables from such a file
  --profile-summary DIR       markdown tables from a rocprofv3 output folder
  --calibrate-copy            plain 1 GiB copies (scale for the HBM counters)
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak

# Traffic through the L2-to-fabric interface per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE (one run each, scaled by a plain 1 GiB copy through the library).  A figure is reported only when the
# library launched exactly the kernel the profile was taken with, on the workload it was taken on, with default
# tuning.  (The counters sit between the L2 and the memory side: reads that the Infinity Cache serves are in it.)
MEASURED_TRAFFIC = {
    # (workload, kernel name as the library reports it): (bytes per launch, profile it comes from)
    ("cfg5", "sparbit::tree_kernel<unsigned int __vector(4), 1, 8, 4, true, false, false, 0, false, 8>"):
        (17802687759, "profiles/tree_kernel_cfg4_cfg5.md"),
    ("cfg4", "sparbit::tree_kernel<unsigned int __vector(4), 1, 8, 4, true, false, false, 0, false, 8>"):
        (17645915435, "profiles/tree_kernel_cfg4_cfg5.md"),
    ("p128_b1048580", "sparbit::tree_kernel<unsigned int __vector(4), 1, 8, 2, true, false, true, 0, false, 1>"):
        (20504780901, "profiles/tree_kernel_cfg4_cfg5.md"),
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg5",
                    help="cfg1 .. cfg5, or pP_bB for P ranks with blocks of B bytes (uint8 payload), e.g. p128_b1048580")
    ap.add_argument("--mode", default="auto", choices=["auto", "per_step", "persistent", "dataflow", "tree"])
    ap.add_argument("--skip-context", action="store_true", help="only the headline workload")
    ap.add_argument("--skip-cpu-baseline", action="store_true")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE")
    ap.add_argument("--sweep", metavar="OUT.jsonl", default=None,
                    help="instead of the benchmark: time every schedule over the block-size ladder 1 B .. 1 MiB "
                         "(doubling, as OSU's osu_allgather in the paper's Section IV-A) for process counts on the "
                         "paper's two progressions, one JSON line per case into OUT.jsonl")
    ap.add_argument("--sweep-summary", metavar="IN.jsonl", default=None,
                    help="instead of the benchmark (no GPU needed): markdown tables from a --sweep file")
    ap.add_argument("--profile-summary", metavar="DIR", default=None,
                    help="instead of the benchmark (no GPU needed): markdown tables from the CSV files of a "
                         "rocprofv3 run (--kernel-trace --stats and/or --pmc, --output-format csv) under DIR")
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


def algorithmic_bytes(form, p, B):
    """HBM bytes one call has to move, by the form it is issued in (see the module docstring).
    `form`: "per_step" (also persistent / dataflow: every forward reads what an earlier phase wrote), "tree"
    (a forwarder is read back right after it was written), "tree_doubling" (Recursive Doubling walked in step order),
    "direct" (every slot straight from the send buffer), "copy" (a device-to-device copy of p*p*B bytes)."""
    landed = p * p * B
    if form in ("tree", "direct"):
        return p * B + landed
    if form == "tree_doubling":  # a forwarder is read a whole step after it was written: p/2 - 1 reads per tree
        return p * B + landed + (p // 2 - 1) * p * B if p > 1 else 2 * B
    return 2 * landed


def form_of(kernel_name, algo_label="sparbit"):
    if algo_label == "direct":
        return "direct"
    if algo_label == "memcpy_d2d":
        return "copy"
    if "tree_kernel" in kernel_name:
        flags = tree_kernel_flags(kernel_name)
        # Recursive Doubling walked in step order reads a forwarder a whole step after it was written; with store
        # forms 1 and 4 it is walked like Sparbit's tree (bits of the relative rank reversed) and read back at once
        return "tree_doubling" if flags["walk"] == "doubling" and flags["store"] not in (1, 4) else "tree"
    return "per_step"


def tree_kernel_flags(kernel_name):
    """Template arguments of the tree kernel's name as the library reports it: access type, vectors per lane, loads
    per batch, store form, look-ahead load, per-slot sizes, any-alignment form, walk, teams, wavefronts per gang."""
    args = kernel_name.rstrip(">").split(", ")
    return {"store": int(args[3]), "any_alignment": args[6] == "true",
            "walk": ("sparbit", "doubling", "chain")[int(args[7])], "team": args[8] == "true",
            "gang": int(args[9]) if len(args) > 9 else 1}


def rates(p, B, ms, form):
    """effective = bytes landed / time; model = the form's algorithmic HBM bytes / time and its share of the peak.
    For jobs that fit the last-level caches the model rate is not an HBM rate (cache_resident)."""
    landed = p * p * B
    model = algorithmic_bytes(form, p, B)
    return {"effective_GBps": landed / ms / 1e6, "form": form, "model_bytes": model,
            "model_GBps": model / ms / 1e6, "model_frac": model / ms / 1e6 / HBM_PEAK_GBPS,
            "cache_resident": landed <= (256 << 20)}


# --------------------------------------------------------------------------- CPU oracle legs
def _host_info():
    model, mem_total, avail = "unknown", 0, 0
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
        for line in open("/proc/meminfo"):
            if line.startswith("MemTotal:"):
                mem_total = int(line.split()[1]) * 1024
            if line.startswith("MemAvailable:"):
                avail = int(line.split()[1]) * 1024
    except OSError:
        pass
    return model, mem_total, avail


def cpu_baseline(w):
    """The oracle as it stands (single-threaded C simulation), timed on the same p with smaller blocks, sized from
    a short probe so that each leg costs roughly 10 s: (a) one run on one thread; (b) one run per core at once,
    every thread its own disjoint problem of the same shape (ctypes releases the GIL, so the runs are parallel).
    The simulation is inherently serial (every step needs the whole previous step), so (b) is the way all cores
    can be used without touching it.  `value` is the larger of the two."""
    import numpy as np
    import oracle
    from paper_2109_08751_amd import workloads

    p = w.p
    model, mem_total, avail = _host_info()
    try:
        cores = int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1)
    except ValueError:
        cores = os.cpu_count() or 1
    cores = max(1, min(cores, os.cpu_count() or 1))

    def problem(B, seed):
        send = np.tile(workloads.make_send_raw(p, min(B, 4096), seed), (1, max(B // 4096, 1)))[:, :B].copy()
        recv = np.full((p, p, B), workloads.POISON, dtype=np.uint8)
        return send, recv

    def run(send, recv):
        B = send.shape[1]
        t = time.perf_counter()
        oracle.allgather(oracle.SPARBIT, p, B, send, recv)
        dt = time.perf_counter() - t
        assert (recv[p - 1, 0] == send[0]).all() and (recv[0, p - 1] == send[p - 1]).all()
        return dt

    B = max(16, min(w.block_bytes, 4096))
    dt = run(*problem(B, 1))
    rate = p * p * B / dt
    target = max(B, min(w.block_bytes, int(rate * 10.0 / (p * p))))
    Bs = 1 << (target.bit_length() - 1)
    # the oracle holds the receive buffers plus a mailbox of up to half their size
    while Bs > B and 2 * p * p * Bs > max(avail // 2, 1 << 30):
        Bs >>= 1
    if Bs > B:
        dt, B = run(*problem(Bs, 1)), Bs
    single = {"GBps": p * p * B / dt / 1e9, "seconds": dt, "block_bytes": B}

    # all cores: the same problem size per thread unless memory says otherwise
    Bm = B
    while Bm > 16 and cores * 2 * p * p * Bm > max(avail // 2, 1 << 30):
        Bm >>= 1
    probs = [problem(Bm, 2 + i) for i in range(cores)]
    times = [0.0] * cores

    def worker(i):
        times[i] = run(*probs[i])

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(cores)]
    t0 = time.perf_counter()
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    wall = time.perf_counter() - t0
    multi = {"GBps": cores * p * p * Bm / wall / 1e9, "seconds": wall, "block_bytes": Bm, "threads": cores}
    best_multi = multi["GBps"] >= single["GBps"]
    return {"value": multi["GBps"] if best_multi else single["GBps"], "unit": "GB/s",
            "cores": cores if best_multi else 1, "kind": "oracle",
            "single_thread": single, "all_cores": multi,
            "host": {"cpu_model": model, "nproc": os.cpu_count(), "mem_total_GiB": round(mem_total / 2**30, 1)},
            "sample": f"Sparbit oracle, p={p}, blocks of {Bm} B instead of {w.block_bytes} B "
                      f"(recv {p * p * Bm / 2**20:.0f} MiB per problem), one pass; the simulation is serial, so the "
                      f"all-cores figure is {cores} independent problems of that shape run at once, one per thread "
                      f"(aggregate bytes landed / wall time); single thread: {single['GBps']:.2f} GB/s on blocks of "
                      f"{B} B"}


# --------------------------------------------------------------------------- block-size ladder
def sweep(torch, sb, workloads, stream, path):
    """Latency/bandwidth ladder in the shape of the paper's test matrix (Section IV-A): block sizes 1 B .. 1 MiB by
    doubling; p from the even/power-of-two progression (8, 16, ..., 256) and the odd one (5, 13, ..., 253), thinned.
    Sparbit is timed as AUTO picks it and as one launch per step; power-of-two p with 4 and 16 KiB blocks also
    through Allgatherv with rows padded by 128 and 256 bytes (same blocks, receive rows no longer a power of two)."""
    import numpy as np
    dev = torch.device("cuda:0")
    ps = [8, 16, 32, 64, 128, 256, 5, 13, 29, 61, 125, 253]
    sizes = [1 << k for k in range(0, 21)]
    if os.environ.get("SPARBIT_SWEEP_PS"):  # a subset, e.g. "128,256"
        ps = [int(x) for x in os.environ["SPARBIT_SWEEP_PS"].split(",")]
    if os.environ.get("SPARBIT_SWEEP_SIZES"):
        sizes = [int(x) for x in os.environ["SPARBIT_SWEEP_SIZES"].split(",")]
    off_grid_bases = [1 << 10, 1 << 14, 1 << 18, 1 << 20]
    if os.environ.get("SPARBIT_SWEEP_OFF_GRID_BASES") is not None:  # "" = none
        off_grid_bases = [int(x) for x in os.environ["SPARBIT_SWEEP_OFF_GRID_BASES"].split(",") if x]
    algos = [("sparbit", sb.SPARBIT, sb.MODE_AUTO), ("sparbit_per_step", sb.SPARBIT, sb.MODE_PER_STEP),
             ("ring", sb.RING, sb.MODE_AUTO), ("recursive_doubling", sb.RECURSIVE_DOUBLING, sb.MODE_AUTO),
             ("recursive_doubling_per_step", sb.RECURSIVE_DOUBLING, sb.MODE_PER_STEP),
             ("bruck", sb.BRUCK, sb.MODE_AUTO), ("direct", sb.DIRECT, sb.MODE_AUTO)]
    n = 0
    with open(path, "w") as out:
        def emit(p, B, label, t, ok, **extra):
            nonlocal n
            out.write(json.dumps({"p": p, "block_bytes": B, "algo": label, "ok": ok,
                                  "avg_us": t["avg_ms"] * 1e3, "min_us": t["min_ms"] * 1e3,
                                  "max_us": t["max_ms"] * 1e3,
                                  "effective_GBps": p * p * B / t["avg_ms"] / 1e6, **extra}) + "\n")
            out.flush()
            n += 1

        for p in ps:
            for B in sizes:
                if p * p * B > (32 << 30):
                    continue
                send = torch.randint(0, 256, (p, B), dtype=torch.uint8, device=dev)
                recv = torch.full((p, p, B), workloads.POISON, dtype=torch.uint8, device=dev)
                for label, algo, md in algos:
                    if algo == sb.RECURSIVE_DOUBLING and p & (p - 1):
                        continue
                    fn = lambda: sb.sparbit_allgather_mode(send, recv, p, B, algo, md, stream)
                    t = time_calls(torch, fn, stream, 3, 10)
                    ok = bool(torch.equal(recv, send.unsqueeze(0).expand(p, p, B))) if p * p * B <= (1 << 28) \
                        else bool(torch.equal(recv[p - 1], send))
                    emit(p, B, label, t, ok)
                    recv.fill_(workloads.POISON)
                    torch.cuda.synchronize()
                del send, recv
                if p in (128, 256) and B in (4096, 16384):
                    for pad in (128, 256):
                        row = p * B + pad
                        counts = np.full(p, B, dtype=np.uint64)
                        displs = np.arange(p, dtype=np.uint64) * B
                        s_ = torch.randint(0, 256, (row,), dtype=torch.uint8, device=dev)
                        r_ = torch.full((p, row), workloads.POISON, dtype=torch.uint8, device=dev)
                        for label, algo, tree in (("sparbit_padded_rows", sb.SPARBIT, 1),
                                                  ("sparbit_per_step_padded_rows", sb.SPARBIT, 0),
                                                  ("recursive_doubling_padded_rows", sb.RECURSIVE_DOUBLING, 1)):
                            sb.sparbit_tune("tree_auto", tree)  # 0: the per-step kernels for blocks of given offsets
                            sb.sparbit_tune("hybrid_max_items", 512 if tree else 0)
                            fn = lambda: sb.sparbit_allgatherv(s_, r_, p, counts, displs, row, algo, stream)
                            t = time_calls(torch, fn, stream, 3, 10)
                            sb.sparbit_tune("tree_auto", 1)
                            sb.sparbit_tune("hybrid_max_items", 512)
                            ok = bool(torch.equal(r_[p - 1, :p * B], s_[:p * B]))
                            emit(p, B, label, t, ok, row_pad=pad)
                            with torch.cuda.stream(stream):
                                r_.fill_(workloads.POISON)
                            torch.cuda.synchronize()
                        del s_, r_
            # Block sizes off the 16-byte / 128-byte grid (the paper's ladder has powers of two only; MPI counts are
            # arbitrary): Sparbit as AUTO issues it, per step, and the two schedules that share its launch count.
            for base in off_grid_bases:
                for extra in (1, 4, 16):
                    B = base + extra
                    if p * p * B > (32 << 30):
                        continue
                    send = torch.randint(0, 256, (p, B), dtype=torch.uint8, device=dev)
                    recv = torch.full((p, p, B), workloads.POISON, dtype=torch.uint8, device=dev)
                    for label, algo, md in algos:
                        if label in ("direct", "recursive_doubling_per_step") or (algo == sb.RECURSIVE_DOUBLING and p & (p - 1)):
                            continue
                        fn = lambda: sb.sparbit_allgather_mode(send, recv, p, B, algo, md, stream)
                        t = time_calls(torch, fn, stream, 3, 10)
                        ok = bool(torch.equal(recv, send.unsqueeze(0).expand(p, p, B))) if p * p * B <= (1 << 28) \
                            else bool(torch.equal(recv[p - 1], send))
                        emit(p, B, label, t, ok, off_grid=True, kernel=sb.sparbit_last_launch_info()[0],
                             rows_on_lines=(p * B) % 128 == 0)
                        recv.fill_(workloads.POISON)
                        torch.cuda.synchronize()
                    del send, recv
            print(f"sweep: p={p} done ({n} cases)", file=sys.stderr, flush=True)
            torch.cuda.empty_cache()
    return n


def sweep_summary(path):
    """Markdown from a --sweep file: per p the fastest schedule at every block size, Sparbit's times, and its ratio to
    Recursive Doubling (power-of-two p) and to its own per-step form."""
    rows = [json.loads(l) for l in open(path)]
    assert all(r["ok"] for r in rows), "a case of the sweep failed its result check"
    by = collections.defaultdict(dict)
    off = collections.defaultdict(dict)
    for r in rows:
        if r.get("off_grid"):
            off[(r["p"], r["block_bytes"])][r["algo"]] = r
            continue
        if "row_pad" in r:
            by[(r["p"], r["block_bytes"])][f"{r['algo']}+{r['row_pad']}"] = r["avg_us"]
        else:
            by[(r["p"], r["block_bytes"])][r["algo"]] = r["avg_us"]
    ps = sorted({k[0] for k in by})
    sizes = sorted({k[1] for k in by})
    schedules = ("sparbit", "ring", "recursive_doubling", "bruck")  # the paper's contenders; DIRECT is no schedule
    out = [f"Cases: {len(rows)}; every result checked.  Times are averages of 10 calls after 3 warm-up calls, in "
           f"microseconds.\n"]
    wins = collections.Counter()
    out.append("## Fastest schedule per (p, block size)  (S = Sparbit, R = Ring, D = Recursive Doubling, B = Bruck)\n")
    out.append("| p \\ bytes | " + " | ".join(_size_label(s) for s in sizes) + " |")
    out.append("|---|" + "---|" * len(sizes))
    letter = {"sparbit": "S", "ring": "R", "recursive_doubling": "D", "bruck": "B"}
    for p in ps:
        cells = []
        for s in sizes:
            c = by.get((p, s))
            if not c:
                cells.append("")
                continue
            best = min((a for a in schedules if a in c), key=lambda a: c[a])
            wins[best] += 1
            cells.append(letter[best])
        out.append(f"| {p} | " + " | ".join(cells) + " |")
    out.append("\nCells won: " + ", ".join(f"{a} {wins[a]}" for a in schedules) + f" of {sum(wins.values())}.\n")
    out.append("## Sparbit (as AUTO issues it), microseconds per call, and effective GB/s\n")
    out.append("| p \\ bytes | " + " | ".join(_size_label(s) for s in sizes) + " |")
    out.append("|---|" + "---|" * len(sizes))
    for p in ps:
        cells = []
        for s in sizes:
            c = by.get((p, s))
            cells.append("" if not c else f"{c['sparbit']:.0f} ({p * p * s / c['sparbit'] / 1e3:.0f})")
        out.append(f"| {p} | " + " | ".join(cells) + " |")
    out.append("\n## Sparbit AUTO time / Sparbit one-launch-per-step time\n")
    out.append("| p \\ bytes | " + " | ".join(_size_label(s) for s in sizes) + " |")
    out.append("|---|" + "---|" * len(sizes))
    for p in ps:
        cells = []
        for s in sizes:
            c = by.get((p, s))
            cells.append("" if not c or "sparbit_per_step" not in c else f"{c['sparbit'] / c['sparbit_per_step']:.2f}")
        out.append(f"| {p} | " + " | ".join(cells) + " |")
    out.append("\n## Sparbit time / Recursive Doubling time (p a power of two)\n")
    out.append("| p \\ bytes | " + " | ".join(_size_label(s) for s in sizes) + " |")
    out.append("|---|" + "---|" * len(sizes))
    for p in ps:
        if p & (p - 1):
            continue
        cells = []
        for s in sizes:
            c = by.get((p, s))
            cells.append("" if not c or "recursive_doubling" not in c else f"{c['sparbit'] / c['recursive_doubling']:.2f}")
        out.append(f"| {p} | " + " | ".join(cells) + " |")
    out.append("\n## Sparbit time / Ring time\n")
    out.append("| p \\ bytes | " + " | ".join(_size_label(s) for s in sizes) + " |")
    out.append("|---|" + "---|" * len(sizes))
    for p in ps:
        cells = []
        for s in sizes:
            c = by.get((p, s))
            cells.append("" if not c or "ring" not in c else f"{c['sparbit'] / c['ring']:.2f}")
        out.append(f"| {p} | " + " | ".join(cells) + " |")
    out.append("\n## Recursive Doubling as AUTO issues it (tree form) / one launch per step\n")
    out.append("| p \\ bytes | " + " | ".join(_size_label(s) for s in sizes) + " |")
    out.append("|---|" + "---|" * len(sizes))
    for p in ps:
        if p & (p - 1):
            continue
        cells = []
        for s in sizes:
            c = by.get((p, s))
            ok = c and "recursive_doubling" in c and "recursive_doubling_per_step" in c
            cells.append(f"{c['recursive_doubling'] / c['recursive_doubling_per_step']:.2f}" if ok else "")
        out.append(f"| {p} | " + " | ".join(cells) + " |")
    padded = [(k, c) for k, c in sorted(by.items()) if any("+" in a for a in c)]
    if padded:
        out.append("\n## Power-of-two p, 4 and 16 KiB blocks: packed rows against rows padded by 128 / 256 bytes (Allgatherv)\n")
        out.append("| p | bytes | Sparbit AUTO | Sparbit per step | Recursive Doubling | Sparbit AUTO +128 | Sparbit AUTO +256 | "
                   "Sparbit per step +128 | Sparbit per step +256 | Rec. Doubling +128 | Rec. Doubling +256 |")
        out.append("|---|---|---|---|---|---|---|---|---|---|---|")
        for (p, s), c in padded:
            g = lambda a: f"{c[a]:.0f}" if a in c else ""
            out.append(f"| {p} | {s} | {g('sparbit')} | {g('sparbit_per_step')} | {g('recursive_doubling')} | "
                       f"{g('sparbit_padded_rows+128')} | {g('sparbit_padded_rows+256')} | "
                       f"{g('sparbit_per_step_padded_rows+128')} | {g('sparbit_per_step_padded_rows+256')} | "
                       f"{g('recursive_doubling_padded_rows+128')} | {g('recursive_doubling_padded_rows+256')} |")
    if off:
        out.append("\n## Block sizes off the 16-byte / 128-byte grid: microseconds per call\n")
        out.append("Rows on lines: p * bytes is a multiple of 128, so every rank's receive buffer lies the same way "
                   "relative to the 128-byte lines.  Form: what AUTO launched (tree* = the tree kernel's any-alignment "
                   "form, tree = its other forms, steps = one launch per step, flow = dataflow launches).\n")
        out.append("| p | bytes | rows on lines | form | Sparbit AUTO | Sparbit per step | AUTO / per step | Recursive Doubling | Ring | Bruck |")
        out.append("|---|---|---|---|---|---|---|---|---|---|")
        for (p, s), c in sorted(off.items()):
            k = c["sparbit"]["kernel"]
            form = ("tree*" if tree_kernel_flags(k)["any_alignment"] else "tree") if "tree_kernel" in k else \
                "flow" if "dataflow" in k else "steps"
            g = lambda a: f"{c[a]['avg_us']:.0f}" if a in c else ""
            base = 1 << (s.bit_length() - 1)
            out.append(f"| {p} | {_size_label(base)}+{s - base} | {'yes' if c['sparbit']['rows_on_lines'] else 'no'} | {form} | "
                       f"{g('sparbit')} | {g('sparbit_per_step')} | "
                       f"{c['sparbit']['avg_us'] / c['sparbit_per_step']['avg_us']:.2f} | {g('recursive_doubling')} | {g('ring')} | {g('bruck')} |")
    return "\n".join(out) + "\n"


def _size_label(s):
    return f"{s >> 20}M" if s >= 1 << 20 else f"{s >> 10}K" if s >= 1 << 10 else str(s)


# --------------------------------------------------------------------------- rocprofv3 CSV reduction
def profile_summary(folder):
    """Markdown from the CSV files rocprofv3 leaves under `folder` (searched recursively; the runs of one workload
    are expected side by side in sub-folders): the kernel statistics, then one table per kernel that joins, per grid
    size, the mean duration from the kernel trace with the mean of every counter collected for that kernel and
    grid size in any of the runs.  Kernel names are cut after their template arguments; only kernels of this library
    are listed in the joined tables."""
    def short(name):
        name = name.replace("void ", "")
        return name[:name.rindex(">(") + 1] if ">(" in name else name.split("(")[0]

    out = []
    for path in sorted(glob.glob(os.path.join(folder, "**", "*kernel_stats.csv"), recursive=True)):
        out.append(f"### {os.path.relpath(path, folder)}\n")
        out.append("| Name | Calls | TotalDurationNs | AverageNs | Percentage | MinNs | MaxNs |\n|---|---|---|---|---|---|---|")
        for r in csv.DictReader(open(path)):
            out.append(f"| {short(r['Name'])} | {r['Calls']} | {r['TotalDurationNs']} | {float(r['AverageNs']):.1f} | "
                       f"{r['Percentage']} | {r['MinNs']} | {r['MaxNs']} |")
        out.append("")
    durations = collections.defaultdict(list)   # (kernel, threads) -> ns
    counters = collections.defaultdict(lambda: collections.defaultdict(list))  # (kernel, threads) -> counter -> values
    for path in sorted(glob.glob(os.path.join(folder, "**", "*kernel_trace.csv"), recursive=True)):
        for r in csv.DictReader(open(path)):
            grid = int(r["Grid_Size_X"]) * int(r["Grid_Size_Y"]) * int(r["Grid_Size_Z"])
            durations[(short(r["Kernel_Name"]), grid)].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    for path in sorted(glob.glob(os.path.join(folder, "**", "*counter_collection.csv"), recursive=True)):
        for r in csv.DictReader(open(path)):
            counters[(short(r["Kernel_Name"]), int(r["Grid_Size"]))][r["Counter_Name"]].append(float(r["Counter_Value"]))
    kernels = sorted({k for k, _ in list(durations) + list(counters) if k.startswith("sparbit::")})
    for kernel in kernels:
        names = sorted({c for (k, _), cs in counters.items() if k == kernel for c in cs})
        grids = sorted({g for k, g in list(durations) + list(counters) if k == kernel})
        out.append(f"### `{kernel}`: per grid size (threads), mean duration over the traced launches and mean counter "
                   f"value per dispatch\n")
        out.append("| threads | traced launches | mean us | min us | max us |" + "".join(f" {c} |" for c in names))
        out.append("|---|---|---|---|---|" + "---|" * len(names))
        for g in grids:
            v = durations.get((kernel, g), [])
            t = f"{len(v)} | {sum(v) / len(v) / 1e3:.1f} | {min(v) / 1e3:.1f} | {max(v) / 1e3:.1f}" if v else "0 | | | "
            cs = counters.get((kernel, g), {})
            out.append(f"| {g} | {t} |" + "".join(f" {sum(cs[c]) / len(cs[c]):.1f} |" if c in cs else " |" for c in names))
        out.append("")
    return "\n".join(out) + "\n"


# --------------------------------------------------------------------------- the benchmark
def main():
    args = parse_args()
    if args.sweep_summary:
        sys.stdout.write(sweep_summary(args.sweep_summary))
        return
    if args.profile_summary:
        sys.stdout.write(profile_summary(args.profile_summary))
        return
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (all virtual ranks share one HBM); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    from paper_2109_08751_amd import workloads
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
    plain_benchmark = not (args.sweep or args.calibrate_copy)
    # The CPU leg runs first, while nothing of the GPU is initialised in this process.
    cpu = cpu_baseline(w) if plain_benchmark and not args.skip_cpu_baseline else None

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    import paper_2109_08751_amd as sb

    for kv in args.tune:
        k, v = kv.split("=")
        sb.sparbit_tune(k, int(v))
    mode = {"auto": sb.MODE_AUTO, "per_step": sb.MODE_PER_STEP, "persistent": sb.MODE_PERSISTENT,
            "dataflow": sb.MODE_DATAFLOW, "tree": sb.MODE_TREE}[args.mode]
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
                          "ok": bool(torch.equal(src, dst)), "kernel": sb.sparbit_last_launch_info()[0], **t,
                          "copy_GBps": 2 * nbytes / t["avg_ms"] / 1e6}))
        return
    p, B = w.p, w.block_bytes

    # ---- headline: timed region of exactly --steps calls
    d_send = make_device_send(torch, w, dev)
    d_recv = torch.full((p, p, B), workloads.POISON, dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    call = lambda: sb.sparbit_allgather_mode(d_send, d_recv, p, B, sb.SPARBIT, mode, stream)
    head = time_calls(torch, call, stream, args.warmup, args.steps)
    kernel, launches = sb.sparbit_last_launch_info()  # what the library's selection rules launched for this call
    assert sb.sparbit_barrier_timeouts(stream) == 0
    ok = all(bool(torch.equal(d_recv[r], d_send)) for r in (0, p // 2, p - 1))
    if not ok:
        print("bench.py: result check failed", file=sys.stderr)
        sys.exit(1)
    form = form_of(kernel)
    r = rates(p, B, head["avg_ms"], form)
    nsteps = sb.Plan(p).num_steps
    traffic = MEASURED_TRAFFIC.get((w.name, kernel)) if not args.tune else None
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
        "roofline": {"bound": "hbm", "achieved": r["model_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": r["model_frac"],
                     "traffic": traffic[0] if traffic else None,
                     "traffic_source": traffic[1] if traffic else None,
                     "kernel": kernel, "form": form,
                     "launches_per_call": launches,
                     "algorithmic_bytes_per_launch": r["model_bytes"] / launches,
                     "avg_launch_ms": head["avg_ms"] / launches,
                     "note": "achieved = algorithmic HBM bytes per launch / average launch duration, the latter from "
                             "HIP events on the launch stream over the timed region (launch gaps included).  "
                             "Algorithmic bytes per call: one launch per step 2*p*p*B (a forwarded byte is read "
                             "from HBM and written to HBM); tree kernel p*B + p*p*B (a wavefront forwards what it "
                             "wrote itself, so only the send buffer has to be read from HBM).  On the 2*p*p*B "
                             "count this call moves %.0f GB/s." % (2 * p * p * B / head["avg_ms"] / 1e6)},
    }

    # ---- per-step durations of the headline workload (outside the timed region): HIP events around
    # sparbit_allgather_steps(s, s), the form with one launch per step
    with torch.cuda.stream(stream):
        d_recv.fill_(workloads.POISON)
        per_step = []
        for rep in range(3):
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(nsteps + 2)]
            evs[0].record(stream)
            for s in range(-1, nsteps):
                sb.sparbit_allgather_steps(d_send, d_recv, p, B, sb.SPARBIT, s, s, stream)
                evs[s + 2].record(stream)
            stream.synchronize()
            per_step = [evs[i].elapsed_time(evs[i + 1]) for i in range(nsteps + 1)]  # the last repetition is kept
    plan = sb.Plan(p)
    out["per_step_ms"] = [{"step": s, "distance": None if s < 0 else plan.step(s)["distance"],
                           "blocks_per_rank": 1 if s < 0 else plan.step(s)["nblocks"],
                           "ms": per_step[s + 1],
                           "hbm_GBps": 2 * p * (1 if s < 0 else plan.step(s)["nblocks"]) * B / per_step[s + 1] / 1e6}
                          for s in range(-1, nsteps)]
    plan.close()
    del d_recv

    # ---- context: other configs, other schedules, copy ceilings
    if not args.skip_context:
        per = {}
        for name in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5"):
            wc = workloads.WORKLOADS[name]
            pc, Bc = wc.p, wc.block_bytes
            s_ = d_send if name == w.name else make_device_send(torch, wc, dev)
            r_ = torch.full((pc, pc, Bc), workloads.POISON, dtype=torch.uint8, device=dev)
            torch.cuda.synchronize()
            row = {"p": pc, "block_bytes": Bc}
            algos = [("sparbit", sb.SPARBIT, sb.MODE_AUTO), ("sparbit_per_step", sb.SPARBIT, sb.MODE_PER_STEP),
                     ("direct", sb.DIRECT, sb.MODE_AUTO)]
            if name in ("cfg1", "cfg2", "cfg3"):
                algos += [("sparbit_dataflow", sb.SPARBIT, sb.MODE_DATAFLOW)]
            if name in ("cfg2", "cfg3", "cfg4", "cfg5"):
                algos += [("bruck", sb.BRUCK, sb.MODE_AUTO)]
                if pc & (pc - 1) == 0:
                    algos += [("recursive_doubling", sb.RECURSIVE_DOUBLING, sb.MODE_AUTO)]
            algos += [("ring", sb.RING, sb.MODE_AUTO)]
            for label, algo, md in algos:
                fn = lambda a=algo, m=md: sb.sparbit_allgather_mode(s_, r_, pc, Bc, a, m, stream)
                t = time_calls(torch, fn, stream, 5, 20)
                kname, nl = sb.sparbit_last_launch_info()
                row[label] = {**t, **rates(pc, Bc, t["avg_ms"], form_of(kname, "direct" if algo == sb.DIRECT else label)),
                              "kernel": kname, "launches_per_call": nl}
                if algo == sb.BRUCK:  # the rotated working buffer doubles the traffic
                    row[label]["model_bytes"] *= 2
                    row[label]["model_GBps"] *= 2
                    row[label]["model_frac"] *= 2
                good = bool(torch.equal(r_[pc - 1], s_))
                row[label]["ok"] = good
                with torch.cuda.stream(stream):
                    r_.fill_(workloads.POISON)
                torch.cuda.synchronize()
            if name == w.name:  # the headline's own roofline block for the other large configuration is below
                row["sparbit"]["headline"] = True
            if name in ("cfg4", "cfg5") and name != w.name:
                c = row["sparbit"]
                c["roofline"] = {"bound": "hbm", "achieved": c["model_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                 "frac": c["model_frac"], "kernel": c["kernel"], "form": c["form"],
                                 "launches_per_call": c["launches_per_call"],
                                 "algorithmic_bytes_per_launch": c["model_bytes"] / c["launches_per_call"],
                                 "avg_launch_ms": c["avg_ms"] / c["launches_per_call"],
                                 "traffic": (MEASURED_TRAFFIC.get((name, c["kernel"])) or (None,))[0]}
            # ceiling: the runtime's device-to-device memcpy of the same p*p*B bytes
            dst = torch.empty_like(r_)
            t = time_calls(torch, lambda: dst.copy_(r_, non_blocking=True), stream, 3, 10)
            row["memcpy_d2d"] = {**t, **rates(pc, Bc, t["avg_ms"], "copy")}
            # floor: PyTorch's fill kernel over the same receive buffers (every delivered byte written once, nothing read)
            t = time_calls(torch, lambda: dst.fill_(0), stream, 2, 8)
            row["fill"] = {**t, "write_GBps": pc * pc * Bc / t["avg_ms"] / 1e6,
                           "frac_of_peak": pc * pc * Bc / t["avg_ms"] / 1e6 / HBM_PEAK_GBPS,
                           "sparbit_over_fill": row["sparbit"]["avg_ms"] / t["avg_ms"]}
            per[name] = row
            del r_, dst, s_
            torch.cuda.empty_cache()
        # Ceilings through the library's own kernels.  Read + write: a linear 4 GiB copy (p = 1: the own-block placement
        # of one block) through the per-step kernel.  Write only: DIRECT on p = 64, 256 KiB blocks (1 GiB written, the
        # 16 MiB send buffer stays in cache), which is what a form that reads nothing back from HBM could reach.
        nbytes = 4 << 30
        src = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device=dev)
        dst = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
        torch.cuda.synchronize()
        t = time_calls(torch, lambda: sb.sparbit_allgather_mode(src, dst, 1, nbytes, sb.SPARBIT, sb.MODE_PER_STEP, stream),
                       stream, 3, 10)
        per["linear_copy_per_step_kernel"] = {"bytes_each_way": nbytes, **t, "kernel": sb.sparbit_last_launch_info()[0],
                                              "read_plus_write_GBps": 2 * nbytes / t["avg_ms"] / 1e6,
                                              "frac_of_peak": 2 * nbytes / t["avg_ms"] / 1e6 / HBM_PEAK_GBPS,
                                              "ok": bool(torch.equal(src, dst))}
        del src, dst
        torch.cuda.empty_cache()
        pw, Bw = 64, 256 << 10
        s_ = torch.randint(0, 256, (pw, Bw), dtype=torch.uint8, device=dev)
        r_ = torch.full((pw, pw, Bw), workloads.POISON, dtype=torch.uint8, device=dev)
        torch.cuda.synchronize()
        t = time_calls(torch, lambda: sb.sparbit_allgather_mode(s_, r_, pw, Bw, sb.DIRECT, sb.MODE_AUTO, stream), stream, 5, 20)
        per["write_only_ceiling_direct_p64_256KiB"] = {"bytes_written": pw * pw * Bw, **t,
                                                       "kernel": sb.sparbit_last_launch_info()[0],
                                                       "write_GBps": pw * pw * Bw / t["avg_ms"] / 1e6,
                                                       "frac_of_peak": pw * pw * Bw / t["avg_ms"] / 1e6 / HBM_PEAK_GBPS,
                                                       "ok": bool(torch.equal(r_[pw - 1], s_))}
        del s_, r_
        torch.cuda.empty_cache()
        # Allgatherv on a cfg4-shaped job: 128 ranks, block sizes spread over 0.5 .. 1.5 MiB (mean 1 MiB), at three
        # granularities: 4 KiB (every block on whole 128-byte lines), 4 bytes and 1 byte.  The last two with rows as
        # long as the blocks need (the rows then lie differently relative to the lines: realigning kernel, one launch
        # per step) and with rows rounded up to whole lines to 1 KiB or to 64 KiB (any-alignment tree form, one launch; in rows a multiple of 64 KiB in gangs).
        import numpy as np
        pv = 128
        for label, grain, row_grain in (("allgatherv_p128_0.5-1.5MiB", 4096, 1),
                                        ("allgatherv_p128_0.5-1.5MiB_grain4B", 4, 1),
                                        ("allgatherv_p128_0.5-1.5MiB_grain1B", 1, 1),
                                        ("allgatherv_p128_0.5-1.5MiB_grain4B_rows128", 4, 128),
                                        ("allgatherv_p128_0.5-1.5MiB_grain1B_rows128", 1, 128),
                                        ("allgatherv_p128_0.5-1.5MiB_grain1B_rows1024", 1, 1024),
                                        ("allgatherv_p128_0.5-1.5MiB_grain1B_rows65536", 1, 65536)):
            rng = np.random.default_rng(workloads.DEFAULT_SEED)
            counts = (rng.integers(512 << 10, (1536 << 10) + 1, pv) // grain * grain).astype(np.uint64)
            displs = np.concatenate([[0], np.cumsum(counts[:-1])]).astype(np.uint64)
            moved = int(counts.sum())
            row = (moved + row_grain - 1) // row_grain * row_grain
            s_ = torch.randint(0, 256, (row,), dtype=torch.uint8, device=dev)
            r_ = torch.full((pv, row), workloads.POISON, dtype=torch.uint8, device=dev)
            torch.cuda.synchronize()
            t = time_calls(torch, lambda: sb.sparbit_allgatherv(s_, r_, pv, counts, displs, row, sb.SPARBIT, stream),
                           stream, 3, 10)
            per[label] = {
                "p": pv, "row_bytes": row, "block_bytes_per_rank": moved, **t,
                "effective_GBps": pv * moved / t["avg_ms"] / 1e6,
                "kernel": sb.sparbit_last_launch_info()[0],
                "ok": bool(torch.equal(r_[pv - 1][:moved], s_[:moved]))}
            vform = form_of(per[label]["kernel"])
            vbytes = moved + pv * moved if vform == "tree" else 2 * pv * moved
            per[label].update({"form": vform, "model_bytes": vbytes, "model_GBps": vbytes / t["avg_ms"] / 1e6,
                               "model_frac": vbytes / t["avg_ms"] / 1e6 / HBM_PEAK_GBPS})
            del s_, r_
            torch.cuda.empty_cache()
        # Equal blocks off the 16-byte grid: cfg4's shape with 4 more bytes per block (rows a multiple of 128 bytes
        # apart: any-alignment tree form), and the same blocks on 125 ranks (rows off the lines: realigning kernel)
        for label, pu, Bu in (("sparbit_p128_1MiB+4B", 128, (1 << 20) + 4), ("sparbit_p125_1MiB+4B", 125, (1 << 20) + 4)):
            s_ = torch.randint(0, 256, (pu, Bu), dtype=torch.uint8, device=dev)
            r_ = torch.full((pu, pu, Bu), workloads.POISON, dtype=torch.uint8, device=dev)
            torch.cuda.synchronize()
            t = time_calls(torch, lambda: sb.sparbit_allgather_mode(s_, r_, pu, Bu, sb.SPARBIT, sb.MODE_AUTO, stream),
                           stream, 3, 10)
            kname = sb.sparbit_last_launch_info()[0]
            per[label] = {"p": pu, "block_bytes": Bu, **t, **rates(pu, Bu, t["avg_ms"], form_of(kname)),
                          "kernel": kname, "ok": bool(torch.equal(r_[pu - 1], s_))}
            del s_, r_
            torch.cuda.empty_cache()
        out["per_config"] = per
        assert sb.sparbit_barrier_timeouts(stream) == 0

    if cpu is not None:
        out["cpu_baseline"] = cpu
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
