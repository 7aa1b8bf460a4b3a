#!/usr/bin/env python3
"""Benchmark of the CSD verification hot path on one MI355X.

A step is one csd_verify call on one batch: ONE kernel launch that streams all B*(k+1) logit rows (softmax
normaliser, lowest-id argmax) and, in the same grid, runs the per-sequence verification loop (draft
probability, memory lookup, gate, accepted-prefix scan) and the memory updates.  Logits are synthetic (seeded
generator, see gen/), already resident in HBM, and replayed from a ring of distinct steps larger than the
last-level cache (>= 1 GiB, >= 4 steps) so that every step's rows come from HBM.  The calls go through the
binding's prepared form (arguments checked and marshalled once per ring entry; each step is then the C call alone).

Every timed loop is preceded by an untimed ramp of fixed duration (RAMP_S of the same launches) and then by
the `--warmup` steps: after an idle gap this GPU needs 10-15 ms of load before its launch times settle (the
first ~150 launches run 5-10 % slow), which a warm-up of a few steps does not cover.  `steps` and `warmup` are
reported exactly as given.

Prints ONE JSON line: whole-path throughput in verified positions (rows) per second at the headline workload;
`roofline` for the dominant kernel (verify_step_kernel, the whole step) from its average launch duration by
events on the launch stream, next to the streaming pass replayed alone (row_partials_kernel, the same streaming
code without the sequence waves) and a read-only probe with the same loads under three deals of the rows to
workgroups (the fastest is the read ceiling); `config.other_workloads` with the other four workloads and the sampling-temperature path, measured
after the headline; and the CPU oracle's rate on the host cores.

Other modes:
  --path sampled       time csd_verify_sampled at --temperature on the chosen workload (one JSON line)
  --path ocm           rates of the memory maintenance entry points (update, export, merge; one JSON line)
  --pmc-run            a short run for rocprofv3 --pmc: a few steps plus plain device-to-device copies of known
                       size, whose counter readings calibrate the counter unit
  --ingest-pmc F W     read the counter CSVs of a FETCH_SIZE run (F) and a WRITE_SIZE run (W) of --pmc-run
                       and write profiles/traffic_<kernel>.json (bytes per launch, kernel fingerprint)
"""
import argparse
import csv
import ctypes
import glob
import hashlib
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E peak, GB/s
STEP_KERNEL = "verify_step_kernel"
STREAM_KERNEL = "row_partials_kernel"
PROBE_TILE_BYTES = 32768       # the streaming pass (and the probe) move whole 32 KiB tiles
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic_verify_step.json")
COPY_BYTES = 1 << 30           # the calibration copy moves 1 GiB in and 1 GiB out
RAMP_S = 0.05                  # untimed load before every timed loop
OTHER_STEPS, OTHER_WARMUP = 200, 20


def kernel_fingerprint() -> str:
    """Hash of everything that shapes the kernels and their launch plan: stored counter readings apply to one version only."""
    h = hashlib.sha256()
    for rel in ("paper_2604_13634_amd/csrc/csd_verify.hip", "paper_2604_13634_amd/csrc/csd_sampled.hip",
                "paper_2604_13634_amd/csrc/csd_stream.h", "paper_2604_13634_amd/csrc/csd_device.h",
                "paper_2604_13634_amd/csrc/csd_internal.h",
                "paper_2604_13634_amd/csrc/csd_api.hip", "include/csd.h", "paper_2604_13634_amd/build.py"):
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def read_counter(path: str, counter: str):
    """{kernel name: [values per dispatch]} of one counter from rocprofv3's counter_collection CSV(s) under `path`."""
    files = [path] if os.path.isfile(path) else glob.glob(os.path.join(path, "**", "*counter_collection.csv"), recursive=True)
    out = {}
    for fn in files:
        with open(fn, newline="") as f:
            for row in csv.DictReader(f):
                if row.get("Counter_Name") != counter:
                    continue
                out.setdefault(row["Kernel_Name"], []).append(float(row["Counter_Value"]))
    return out


def ingest_pmc(fetch_path: str, write_path: str, workload: str, kernels) -> int:
    """Scale FETCH_SIZE / WRITE_SIZE of the named kernels by what the same counters read for the 1 GiB copy."""
    rec = {}
    if os.path.exists(TRAFFIC_FILE):
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f)
    ent = {"kernel": kernels[0], "kernel_fingerprint": kernel_fingerprint(), "copy_bytes_each_way": COPY_BYTES, "kernels": {}}
    for kname in kernels:
        kent = {}
        total = 0.0
        for name, path in (("FETCH_SIZE", fetch_path), ("WRITE_SIZE", write_path)):
            per_kernel = read_counter(path, name)
            stream = [v for k, vals in per_kernel.items() if kname in k for v in vals]
            # the calibration copies are the largest launches of a copy kernel in the run
            copies = [v for k, vals in per_kernel.items() if "copy" in k.lower() for v in vals]
            if not stream or not copies:
                print("bench.py: no %s readings for %s or the copy in %s" % (name, kname, path), file=sys.stderr)
                return 1
            copy_read = max(copies)
            unit = COPY_BYTES / copy_read                      # bytes per counter unit on this machine
            mean = sum(stream) / len(stream)
            kent[name] = {"kernel_mean_reading": mean, "kernel_launches": len(stream), "copy_reading": copy_read,
                          "bytes_per_unit": unit, "bytes_per_launch": mean * unit}
            total += mean * unit
        kent["hbm_bytes_per_launch"] = total
        ent["kernels"][kname] = kent
    ent["hbm_bytes_per_launch"] = ent["kernels"][kernels[0]]["hbm_bytes_per_launch"]
    rec[workload] = ent
    with open(TRAFFIC_FILE, "w") as f:
        json.dump(rec, f, indent=1, sort_keys=True)
        f.write("\n")
    print(json.dumps(ent))
    return 0


# --------------------------------------------------------------------------------------------- timing helpers
def ramp(fn, seconds=RAMP_S):
    """Untimed: keep launching fn(i) until `seconds` have passed with the GPU busy."""
    import torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    i = 0
    while time.perf_counter() - t0 < seconds:
        for _ in range(50):
            fn(i)
            i += 1
        torch.cuda.synchronize()
    return i


def timed(fn, steps, warmup):
    """ramp, `warmup` untimed launches, then exactly `steps` launches between two synchronisations.
    Returns (wall seconds, milliseconds per launch by events on the launch stream)."""
    import torch
    ramp(fn)
    for i in range(warmup):
        fn(i)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()                                       # events on the stream the kernels are launched on
    for i in range(steps):
        fn(warmup + i)
    e1.record()
    torch.cuda.synchronize()
    return time.perf_counter() - t0, e0.elapsed_time(e1) / steps


def make_ring(w, cfg, ring_bytes, gen_threads, keep_host=0, sampled=False):
    import torch
    from gen.device import to_device_logits
    step_bytes = cfg.bytes_per_step + (cfg.B * cfg.k * cfg.V * cfg.itemsize if sampled else 0)
    n_ring = max(4, int(math.ceil(ring_bytes / step_bytes)))
    ring, host = [], []
    for s in range(n_ring):
        if sampled:
            zp, zq, d, ua, ud = w.sampled_step(s, threads=gen_threads)
            ring.append((to_device_logits(zp), to_device_logits(zq), torch.from_numpy(d).cuda(), torch.from_numpy(ua).cuda(),
                         torch.from_numpy(ud).cuda()))
        else:
            z, d = w.step(s, threads=gen_threads)
            ring.append((to_device_logits(z), torch.from_numpy(d).cuda()))
            if s < keep_host:
                host.append((z, d))
    torch.cuda.synchronize()
    return ring, host


def measure_greedy(cfg, steps, warmup, ring_bytes, gen_threads, full=False, keep_host=0):
    """Times csd_verify on one workload.  full: also the two-batches-in-flight rate, the streaming pass alone and
    the read probe.  Returns (result dict, host copies of the first ring steps)."""
    import numpy as np
    import torch
    from gen import Workload
    from paper_2604_13634_amd import binding as csd

    w = Workload(cfg)
    t_gen = time.perf_counter()
    ring, host = make_ring(w, cfg, ring_bytes, gen_threads, keep_host)
    t_gen = time.perf_counter() - t_gen
    n_ring = len(ring)
    dt = csd.CSD_DTYPE_F32 if cfg.dtype == "f32" else csd.CSD_DTYPE_BF16
    bf = csd.VerifyBuffers.allocate(cfg.B, cfg.k, cfg.V, dt)
    rows, alg_bytes = cfg.rows, cfg.bytes_per_step     # every logit read once; records and outputs are a few KB

    def leg(flags):
        ocm = csd.new_ocm(cfg.capacity)
        # arguments checked and marshalled once per ring entry, as a serving loop would: launch() is the C call alone
        calls = [csd.prepare_verify(z, d, cfg.tau, cfg.lam, ocm, flags, buffers=bf) for z, d in ring]
        fn = lambda i: calls[i % n_ring].launch()
        wall, ev_ms = timed(fn, steps, warmup)
        return wall, ev_ms

    bf.status.zero_()
    wall, ev_ms = leg(csd.CSD_APPLY_UPDATES)
    accept_rate = float(bf.accept_len.float().mean().item()) / max(cfg.k, 1)
    status = bf.status.cpu().numpy().view(np.uint32).tolist()
    wall_no, ev_no = leg(0)
    ms = wall / steps * 1e3
    res = {
        "workload": cfg.name, "B": cfg.B, "k": cfg.k, "V": cfg.V, "logits_storage": cfg.dtype,
        "positions_per_step": rows, "draft_positions_per_step": cfg.B * cfg.k, "tau": cfg.tau, "lambda": cfg.lam,
        "ocm_capacity": cfg.capacity, "steps": steps, "warmup": warmup, "ms_per_step": ms, "us_per_call": ms * 1e3,
        "positions_per_s": rows * steps / wall, "ms_per_step_by_stream_events": ev_ms,
        "positions_per_s_without_ocm_updates": rows * steps / wall_no, "ms_per_step_without_ocm_updates": wall_no / steps * 1e3,
        "logit_bytes_per_step": alg_bytes, "GBps": alg_bytes / (ms * 1e-3) / 1e9,
        "frac_of_hbm_peak": alg_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "ring_steps": n_ring, "ring_bytes": n_ring * alg_bytes, "accept_rate_last_step": accept_rate,
        "status_counters": status, "input_generation_s": t_gen,
    }
    if full:
        # two independent batches in flight (two streams, each with its own buffers and memory): one batch's sequence
        # waves and launch gap overlap the other's streaming
        lanes = []
        for _ in range(2):
            st = torch.cuda.Stream()
            with torch.cuda.stream(st):
                lanes.append((st, csd.VerifyBuffers.allocate(cfg.B, cfg.k, cfg.V, dt), csd.new_ocm(cfg.capacity)))
        torch.cuda.synchronize()

        two_calls = [[csd.prepare_verify(z, d, cfg.tau, cfg.lam, o2, buffers=b2, stream=st) for z, d in ring]
                     for st, b2, o2 in lanes]

        def two(i):
            two_calls[i & 1][i % n_ring].launch()
        ramp(two)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            two(i)
        torch.cuda.synchronize()
        res["positions_per_s_two_batches_in_flight"] = rows * steps / (time.perf_counter() - t0)

        # the streaming pass alone: the same streaming code as its own kernel (no sequence waves in the grid)
        part = csd.csd_row_partials(ring[0][0])
        _, k_ms = timed(lambda i: csd.csd_row_partials(ring[i % n_ring][0], part), steps, warmup)
        res["streaming_pass_alone"] = {"kernel": "%s<%s>" % (STREAM_KERNEL, cfg.dtype), "kernel_ms": k_ms,
                                       "GBps": alg_bytes / (k_ms * 1e-3) / 1e9,
                                       "frac": alg_bytes / (k_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        # read-only probe: the streaming pass's loads and nothing else, dealt to the product's number of workgroups
        # per row and to two other deals (one tile per workgroup, four tiles); the fastest is the ceiling
        probe = ctypes.CDLL(os.path.join(ROOT, "paper_2604_13634_amd", "libcsd_probe.so"))
        probe.csd_probe_read.restype = ctypes.c_int64
        probe.csd_probe_read.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_int64, ctypes.c_int,
                                         ctypes.c_void_p, ctypes.c_void_p]
        sink = torch.zeros(4, dtype=torch.int32, device="cuda")
        nsplit = csd.csd_row_partials_per_row(rows, cfg.V, dt) // 4
        ntiles = max(1, (cfg.V * cfg.itemsize) // PROBE_TILE_BYTES)
        shapes = {}
        for ns in sorted({nsplit, ntiles, (ntiles + 3) // 4}):
            read = [0]

            def pr(i, ns=ns):
                z = ring[i % n_ring][0]
                read[0] = probe.csd_probe_read(z.data_ptr(), z.stride(1) * cfg.itemsize, rows, cfg.V * cfg.itemsize, ns,
                                               sink.data_ptr(), torch.cuda.current_stream().cuda_stream or None)
            pr(0)
            if read[0] > 0:
                _, p_ms = timed(pr, steps, warmup)
                shapes[ns] = {"workgroups_per_row": ns, "bytes_per_launch": read[0], "kernel_ms": p_ms,
                              "GBps": read[0] / (p_ms * 1e-3) / 1e9}
        if shapes:
            best = max(shapes.values(), key=lambda e: e["GBps"])
            res["read_probe"] = dict(best, product_workgroups_per_row=nsplit,
                                     all_deals={str(ns): round(e["GBps"], 1) for ns, e in shapes.items()})
    del ring
    torch.cuda.empty_cache()
    return res, host, w


def measure_sampled(cfg, steps, warmup, ring_bytes, gen_threads, temperature, pmc_run=False):
    """Whole-step timing of csd_verify_sampled on the sampled variant of a workload (target and draft logits,
    uniforms as generated: nothing is compared here, so they are not moved away from decision boundaries)."""
    import numpy as np
    import torch
    from gen.workload import SampledWorkload
    from paper_2604_13634_amd import binding as csd

    w = SampledWorkload(cfg)
    ring, _ = make_ring(w, cfg, 0 if pmc_run else ring_bytes, gen_threads, sampled=True)
    n_ring = len(ring)
    dt = csd.CSD_DTYPE_F32 if cfg.dtype == "f32" else csd.CSD_DTYPE_BF16
    bf = csd.SampledBuffers.allocate(cfg.B, cfg.k, cfg.V, dt)
    ocm = csd.new_ocm(cfg.capacity)

    def step(i):
        zp, zq, d, ua, ud = ring[i % n_ring]
        csd.csd_verify_sampled(zp, zq, d, temperature, ua, ud, cfg.tau, cfg.lam, ocm, buffers=bf)

    if pmc_run:
        for i in range(10):
            step(i)
        torch.cuda.synchronize()
        return None
    wall, ev_ms = timed(step, steps, warmup)
    step_bytes = (cfg.rows + cfg.B * cfg.k) * cfg.V * cfg.itemsize
    # rows the second pass streamed in the last step: two per rejected position, one per bonus draw
    rejected = int((bf.tstar >= 0).sum().item())
    pass2_bytes = (2 * rejected + cfg.B) * cfg.V * cfg.itemsize
    ms = wall / steps * 1e3
    alg = step_bytes + pass2_bytes
    res = {"workload": cfg.name + "+draft_logits", "path": "csd_verify_sampled", "temperature": temperature, "B": cfg.B,
           "k": cfg.k, "V": cfg.V, "logits_storage": cfg.dtype, "positions_per_step": cfg.rows, "steps": steps, "warmup": warmup,
           "ms_per_step": ms, "positions_per_s": cfg.rows * steps / wall, "ms_per_step_by_stream_events": ev_ms,
           "rows_streamed_first_pass": cfg.rows + cfg.B * cfg.k, "rejected_positions_last_step": rejected,
           "first_pass_bytes": step_bytes, "second_pass_bytes_last_step": pass2_bytes, "algorithmic_bytes_per_step": alg,
           "GBps": alg / (ms * 1e-3) / 1e9, "frac_of_hbm_peak": alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "ring_steps": n_ring,
           "status_counters": bf.status.cpu().numpy().view(np.uint32).tolist()}
    del ring
    torch.cuda.empty_cache()
    return res


def measure_ocm() -> dict:
    """Rates of the memory maintenance entry points on a 2^22-slot table (lists generated on the device with torch)."""
    import torch
    from paper_2604_13634_amd import binding as csd

    def rate(fn, n, reps=5):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        return {"entries": n, "ms": ms, "entries_per_s": n / (ms * 1e-3)}

    gen = torch.Generator(device="cuda").manual_seed(1)
    cap = 1 << 22
    n = 1 << 24
    out = {"table_slots": cap}
    d = torch.randint(0, 1 << 18, (n,), generator=gen, device="cuda", dtype=torch.int64)
    uniform = (d << 20) | ((d * 7 + 1) & 0xFFFFF)
    ocm = csd.new_ocm(cap)
    out["update_uniform_over_2^18_pairs"] = rate(lambda: csd.csd_ocm_update(ocm, uniform), n)
    ranks = torch.arange(1, 65, device="cuda", dtype=torch.float64) ** -1.5
    hot_idx = torch.multinomial((ranks / ranks.sum()).float(), n, replacement=True, generator=gen)
    hot = ((hot_idx + 1) << 20) | (hot_idx + 100)
    ocm2 = csd.new_ocm(cap)
    out["update_64_hot_pairs_zipf1.5"] = rate(lambda: csd.csd_ocm_update(ocm2, hot), n)
    distinct = (torch.arange(1 << 20, device="cuda", dtype=torch.int64) << 20) | 5
    ocm3 = csd.new_ocm(cap)
    out["update_2^20_distinct_pairs"] = rate(lambda: (csd.csd_ocm_reset(ocm3), csd.csd_ocm_update(ocm3, distinct)), 1 << 20)
    bufs = (torch.empty(cap, dtype=torch.int64, device="cuda"), torch.empty(cap, dtype=torch.int32, device="cuda"),
            torch.empty(1, dtype=torch.int64, device="cuda"))
    out["export_2^18_pairs"] = rate(lambda: csd.csd_ocm_export(ocm, out=bufs), 1 << 18)
    out["export_2^20_pairs"] = rate(lambda: csd.csd_ocm_export(ocm3, out=bufs), 1 << 20)
    big = csd.new_ocm(1 << 23)
    out["merge_2^18_pairs_into_2^23_slots"] = rate(lambda: csd.csd_ocm_merge(big, ocm), 1 << 18)
    out["reset_2^22_slots"] = rate(lambda: csd.csd_ocm_reset(ocm3), cap)
    return out


def cpu_baseline(w, cfg, host, gen_threads) -> dict:
    """The oracle as it stands, on the host cores, on a bounded sample of the same workload: all cores and one thread."""
    import numpy as np
    from oracle import csd_oracle as O
    cores = min(16, len(os.sched_getaffinity(0)))
    if cfg.bytes_per_step < (64 << 20):          # small workloads: regenerate more steps for a stable number
        extra = min(cfg.steps, max(4, int((256 << 20) // cfg.bytes_per_step)))
        host = [w.step(s, threads=gen_threads) for s in range(extra)]
    O.row_stats(host[0][0][:1])                  # load the library outside the timed part
    passes = 4 if cfg.bytes_per_step >= (64 << 20) else 1      # about 10-30 core-seconds in all
    orc = O.CSDOracle(capacity=cfg.capacity)
    t0 = time.perf_counter()
    for _ in range(passes):
        for z, d in host:
            orc.verify_step(z, d, tau=np.float32(cfg.tau), lam=cfg.lam, threads=cores)
    t_all = time.perf_counter() - t0
    n_all = len(host) * passes
    one = host[:1] if cfg.bytes_per_step >= (64 << 20) else host[:max(1, len(host) // 8)]
    orc1 = O.CSDOracle(capacity=cfg.capacity)
    t0 = time.perf_counter()
    for z, d in one:
        orc1.verify_step(z, d, tau=np.float32(cfg.tau), lam=cfg.lam, threads=1)
    t_one = time.perf_counter() - t0
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return {
        "value": cfg.rows * n_all / t_all, "unit": "positions/s", "cores": cores, "kind": "oracle",
        "sample": "%d steps of %s (%d positions), fp64 oracle, rows split over %d threads, scan and memory serial"
                  % (n_all, cfg.name, cfg.rows * n_all, cores),
        "seconds": t_all,
        "one_thread": {"value": cfg.rows * len(one) / t_one, "unit": "positions/s", "seconds": t_one,
                       "sample": "%d steps (%d positions) on one thread" % (len(one), cfg.rows * len(one))},
        "nproc": os.cpu_count(), "cpus_allowed": len(os.sched_getaffinity(0)), "cpu_model": model,
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4, help="workload index 0..4 (default: the largest, 4)")
    ap.add_argument("--ring-bytes", type=float, default=float(1 << 30), help="minimum bytes of distinct logits in the ring")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true", help="skip config.other_workloads")
    ap.add_argument("--gen-threads", type=int, default=16)
    ap.add_argument("--path", choices=("greedy", "sampled", "ocm"), default="greedy",
                    help="greedy: csd_verify (the headline); sampled: csd_verify_sampled at --temperature; ocm: memory maintenance rates")
    ap.add_argument("--temperature", type=float, default=1.0)
    ap.add_argument("--batch", type=int, help="override the workload's B")
    ap.add_argument("--draft-len", type=int, help="override the workload's k")
    ap.add_argument("--vocab", type=int, help="override the workload's V")
    ap.add_argument("--tau", type=float, help="override the gate threshold")
    ap.add_argument("--lam", type=int, help="override the frequency threshold")
    ap.add_argument("--pmc-run", action="store_true", help="short run for rocprofv3 --pmc (see module docstring)")
    ap.add_argument("--ingest-pmc", nargs=2, metavar=("FETCH", "WRITE"))
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on ONE GPU only (there is no multi-GPU path); use --gpus 1", file=sys.stderr)
        return 2

    from gen import CONFIGS
    cfg = CONFIGS[args.config]
    over = {k: v for k, v in (("B", args.batch), ("k", args.draft_len), ("V", args.vocab), ("tau", args.tau), ("lam", args.lam))
            if v is not None}
    if over:
        import dataclasses
        cfg = dataclasses.replace(cfg, name=cfg.name + "".join("_%s%g" % kv for kv in sorted(over.items())), **over)
    if args.ingest_pmc:
        if args.path == "sampled":
            return ingest_pmc(args.ingest_pmc[0], args.ingest_pmc[1], cfg.name + "+sampled",
                              ("sampled_stream_kernel", "residual_segments_kernel"))
        return ingest_pmc(args.ingest_pmc[0], args.ingest_pmc[1], cfg.name, (STEP_KERNEL,))

    import torch
    torch.cuda.set_device(0)
    metric = "verified draft positions/sec + achieved HBM GB/s (% of peak) of csd_verify"

    if args.path == "ocm":
        print(json.dumps({"metric": "Online Correction Memory maintenance rates", "unit": "entries/s", "n_gpus": 1,
                          "data": "synthetic", "rates": measure_ocm()}))
        return 0

    if args.pmc_run:
        if args.path == "sampled":
            measure_sampled(cfg, 0, 0, 0, args.gen_threads, args.temperature, pmc_run=True)
        else:
            from gen import Workload
            from paper_2604_13634_amd import binding as csd
            ring, _ = make_ring(Workload(cfg), cfg, 0, args.gen_threads)
            dt = csd.CSD_DTYPE_F32 if cfg.dtype == "f32" else csd.CSD_DTYPE_BF16
            bf = csd.VerifyBuffers.allocate(cfg.B, cfg.k, cfg.V, dt)
            ocm = csd.new_ocm(cfg.capacity)
            for i in range(10):
                csd.csd_verify(ring[i % 4][0], ring[i % 4][1], cfg.tau, cfg.lam, ocm, buffers=bf)
        src = torch.empty(COPY_BYTES, dtype=torch.uint8, device="cuda")
        src.random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print("pmc-run done: 10 steps of %s (%s path), 3 copies of %d bytes" % (cfg.name, args.path, COPY_BYTES))
        return 0

    if args.path == "sampled":
        r = measure_sampled(cfg, args.steps, args.warmup, args.ring_bytes, args.gen_threads, args.temperature)
        out = {"metric": metric + "_sampled", "value": r["positions_per_s"], "unit": "positions/s", "n_gpus": 1,
               "steps": args.steps, "warmup": args.warmup, "ms_per_step": r["ms_per_step"], "higher_is_better": True,
               "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic", "config": r,
               "roofline": {"bound": "hbm", "kernel": "whole step (its launches together)", "achieved": r["GBps"],
                            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": r["frac_of_hbm_peak"], "traffic": None,
                            "algorithmic_bytes_per_step": r["algorithmic_bytes_per_step"]}}
        print(json.dumps(out))
        return 0

    # ---- the headline: the whole hot path, memory updates applied
    head, host, w = measure_greedy(cfg, args.steps, args.warmup, args.ring_bytes, args.gen_threads, full=True, keep_host=4)
    k_ms = head["ms_per_step_by_stream_events"]      # one kernel per step: the launch period is the step
    achieved = head["logit_bytes_per_step"] / (k_ms * 1e-3) / 1e9
    traffic, traffic_source = None, None
    if os.path.exists(TRAFFIC_FILE):
        with open(TRAFFIC_FILE) as f:
            ent = json.load(f).get(cfg.name)
        if ent and ent.get("kernel_fingerprint") == kernel_fingerprint():
            traffic = ent["hbm_bytes_per_launch"]
            traffic_source = "profiles/%s @ kernel fingerprint %s (rocprofv3 --pmc runs, not this run)" % (
                os.path.basename(TRAFFIC_FILE), ent["kernel_fingerprint"])
    config = dict(head)
    config.update({"ocm_updates": "applied", "launch": "one kernel launch per step",
                   "arithmetic": "bf16/f32 logits widened to f32; sums f32 per lane, combined in f64; decisions in f64",
                   "ramp_s_before_each_timed_loop": RAMP_S,
                   "whole_path_GBps": head["GBps"], "whole_path_frac_of_hbm_peak": head["frac_of_hbm_peak"]})
    out = {
        "metric": metric, "value": head["positions_per_s"], "unit": "positions/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic", "config": config,
        "roofline": {
            "bound": "hbm", "kernel": "%s<%s> (the whole step)" % (STEP_KERNEL, cfg.dtype), "achieved": achieved,
            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
            "traffic_source": traffic_source, "kernel_ms": k_ms, "algorithmic_bytes_per_launch": head["logit_bytes_per_step"],
            "streaming_pass_alone": head.get("streaming_pass_alone"),
        },
    }
    probe = head.get("read_probe")
    if probe:
        out["roofline"]["read_ceiling_GBps"] = probe["GBps"]
        out["roofline"]["frac_of_read_ceiling"] = achieved / probe["GBps"]
        out["roofline"]["streaming_pass_frac_of_read_ceiling"] = head["streaming_pass_alone"]["GBps"] / probe["GBps"]

    # ---- the other workloads and the sampling-temperature path (after the headline; fixed step counts)
    if not args.no_other_workloads and not over:
        others = {}
        for ci in range(len(CONFIGS)):
            if ci == args.config:
                continue
            r, _, _ = measure_greedy(CONFIGS[ci], OTHER_STEPS, OTHER_WARMUP, args.ring_bytes, args.gen_threads)
            others[CONFIGS[ci].name] = {k: r[k] for k in ("B", "k", "V", "logits_storage", "steps", "warmup", "ms_per_step",
                                                          "us_per_call", "positions_per_s", "ms_per_step_without_ocm_updates",
                                                          "GBps", "frac_of_hbm_peak", "ring_steps")}
        s = measure_sampled(cfg, OTHER_STEPS, OTHER_WARMUP, args.ring_bytes, args.gen_threads, args.temperature)
        others[cfg.name + "_sampled_T%g" % args.temperature] = {k: s[k] for k in (
            "path", "B", "k", "V", "logits_storage", "steps", "warmup", "ms_per_step", "positions_per_s",
            "rejected_positions_last_step", "algorithmic_bytes_per_step", "GBps", "frac_of_hbm_peak", "ring_steps")}
        out["config"]["other_workloads"] = others

    # ---- CPU baseline: the oracle as it stands, on the host cores, on a bounded sample of the same workload
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, cfg, host, args.gen_threads)

    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
