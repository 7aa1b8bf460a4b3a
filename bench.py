#!/usr/bin/env python3
"""Benchmark of the CSD verification hot path on one MI355X.

A step is one csd_verify call on one batch: the streaming pass over all B*(k+1) logit rows, the
per-sequence epilogue (draft probability, memory lookup, gate, accepted-prefix scan) and the
memory updates.  Logits are synthetic (seeded generator, see gen/), already resident in HBM, and
replayed from a ring of distinct steps larger than the last-level cache (>= 1 GiB, >= 4 steps) so
that every step's rows come from HBM.

Prints ONE JSON line: whole-path throughput in verified positions (rows) per second; the achieved HBM
bandwidth of the dominant kernel (the streaming pass, row_partials_kernel) against the 8 TB/s peak, from
its average launch duration measured with events on the launch stream while it is replayed over the same
ring in the launch shape csd_verify uses; and the CPU oracle's rate on the host cores.

Two more modes serve the hardware-counter runs (rocprofv3 --pmc) behind "roofline.traffic":
  --pmc-run            a short run: a few csd_verify steps plus plain device-to-device copies of known
                       size, whose counter readings calibrate the counter unit
  --ingest-pmc F W     read the counter CSVs of a FETCH_SIZE run (F) and a WRITE_SIZE run (W) of --pmc-run
                       and write profiles/traffic_row_partials.json (bytes per launch, kernel fingerprint)
"""
import argparse
import csv
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
STREAM_KERNEL = "row_partials_kernel"
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic_row_partials.json")
COPY_BYTES = 1 << 30           # the calibration copy moves 1 GiB in and 1 GiB out


def kernel_fingerprint() -> str:
    """Hash of the streaming kernel's source and build flags: stored counter readings apply to one version only."""
    h = hashlib.sha256()
    for rel in ("paper_2604_13634_amd/csrc/csd_verify.hip", "paper_2604_13634_amd/csrc/csd_sampled.hip",
                "paper_2604_13634_amd/csrc/csd_device.h",
                "paper_2604_13634_amd/csrc/csd_internal.h", "paper_2604_13634_amd/build.py"):
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


def ingest_pmc(fetch_path: str, write_path: str, workload: str, kernels=(STREAM_KERNEL,)) -> int:
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
            kent[name] = {"stream_mean_reading": mean, "stream_launches": len(stream), "copy_reading": copy_read,
                          "bytes_per_unit": unit, "bytes_per_launch": mean * unit}
            total += mean * unit
        kent["hbm_bytes_per_launch"] = total
        ent["kernels"][kname] = kent
    first = ent["kernels"][kernels[0]]
    ent["FETCH_SIZE"], ent["WRITE_SIZE"], ent["hbm_bytes_per_launch"] = first["FETCH_SIZE"], first["WRITE_SIZE"], first["hbm_bytes_per_launch"]
    rec[workload] = ent
    with open(TRAFFIC_FILE, "w") as f:
        json.dump(rec, f, indent=1, sort_keys=True)
        f.write("\n")
    print(json.dumps(ent))
    return 0


def bench_sampled(args, cfg) -> int:
    """Whole-step timing of csd_verify_sampled on the sampled variant of a workload (target and draft logits,
    uniforms as generated: nothing is compared here, so they are not moved away from decision boundaries)."""
    import numpy as np
    import torch

    from gen.workload import SampledWorkload
    from paper_2604_13634_amd import binding as csd

    from gen.device import to_device_logits

    w = SampledWorkload(cfg)
    step_bytes = (cfg.rows + cfg.B * cfg.k) * cfg.V * cfg.itemsize
    n_ring = max(4, int(math.ceil(args.ring_bytes / step_bytes)))
    if args.pmc_run:
        n_ring = 4
    ring = []
    for s in range(n_ring):
        zp, zq, d, ua, ud = w.sampled_step(s, threads=args.gen_threads)
        ring.append((to_device_logits(zp), to_device_logits(zq), torch.from_numpy(d).cuda(), torch.from_numpy(ua).cuda(),
                     torch.from_numpy(ud).cuda()))
    torch.cuda.synchronize()
    dt = csd.CSD_DTYPE_F32 if cfg.dtype == "f32" else csd.CSD_DTYPE_BF16
    bf = csd.SampledBuffers.allocate(cfg.B, cfg.k, cfg.V, dt)
    ocm = csd.new_ocm(cfg.capacity)

    def step(i):
        zp, zq, d, ua, ud = ring[i % n_ring]
        csd.csd_verify_sampled(zp, zq, d, args.temperature, ua, ud, cfg.tau, cfg.lam, ocm, buffers=bf)

    if args.pmc_run:
        for i in range(10):
            step(i)
        src = torch.empty(COPY_BYTES, dtype=torch.uint8, device="cuda")
        src.random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print("pmc-run done: 10 csd_verify_sampled steps of %s, 3 copies of %d bytes" % (cfg.name, COPY_BYTES))
        return 0
    for i in range(args.warmup):
        step(i)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for i in range(args.steps):
        step(args.warmup + i)
    e1.record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    # rows the second pass streamed in the last step: two per rejected position, one per bonus draw
    rejected = int((bf.tstar >= 0).sum().item())
    pass2_bytes = (2 * rejected + cfg.B) * cfg.V * cfg.itemsize
    ms = elapsed / args.steps * 1e3
    alg = step_bytes + pass2_bytes
    status = bf.status.cpu().numpy().view(np.uint32).tolist()
    out = {
        "metric": "verified draft positions/sec + achieved HBM GB/s (% of peak) of csd_verify_sampled",
        "value": cfg.rows * args.steps / elapsed, "unit": "positions/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg.name + "+draft_logits", "path": "sampled", "temperature": args.temperature, "B": cfg.B,
                   "k": cfg.k, "V": cfg.V, "logits_storage": cfg.dtype, "positions_per_step": cfg.rows,
                   "rows_streamed_first_pass": cfg.rows + cfg.B * cfg.k, "rejected_positions_last_step": rejected,
                   "first_pass_bytes": step_bytes, "second_pass_bytes_last_step": pass2_bytes,
                   "ms_per_step_by_stream_events": e0.elapsed_time(e1) / args.steps, "ring_steps": n_ring,
                   "status_counters": status},
        "roofline": {"bound": "hbm", "kernel": "whole step (five launches)", "achieved": alg / (ms * 1e-3) / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None,
                     "algorithmic_bytes_per_step": alg},
    }
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4, help="workload index 0..4 (default: the largest, 4)")
    ap.add_argument("--ring-bytes", type=float, default=float(1 << 30), help="minimum bytes of distinct logits in the ring")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--gen-threads", type=int, default=16)
    ap.add_argument("--path", choices=("greedy", "sampled"), default="greedy",
                    help="greedy: csd_verify (the headline); sampled: csd_verify_sampled at --temperature")
    ap.add_argument("--temperature", type=float, default=1.0)
    ap.add_argument("--batch", type=int, help="override the workload's B")
    ap.add_argument("--draft-len", type=int, help="override the workload's k")
    ap.add_argument("--vocab", type=int, help="override the workload's V")
    ap.add_argument("--tau", type=float, help="override the gate threshold")
    ap.add_argument("--lam", type=int, help="override the frequency threshold")
    ap.add_argument("--graph", action="store_true",
                    help="greedy path: replay each step from a captured graph instead of launching it (ring capped at 64 steps)")
    ap.add_argument("--pmc-run", action="store_true", help="short run for rocprofv3 --pmc (see module docstring)")
    ap.add_argument("--ingest-pmc", nargs=2, metavar=("FETCH", "WRITE"))
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no multi-GPU path exists); use --gpus 1", file=sys.stderr)
        return 2

    from gen import CONFIGS, Workload
    cfg = CONFIGS[args.config]
    over = {k: v for k, v in (("B", args.batch), ("k", args.draft_len), ("V", args.vocab), ("tau", args.tau), ("lam", args.lam))
            if v is not None}
    if over:
        import dataclasses
        cfg = dataclasses.replace(cfg, name=cfg.name + "".join("_%s%g" % kv for kv in sorted(over.items())), **over)
    if args.ingest_pmc:
        if args.path == "sampled":
            return ingest_pmc(args.ingest_pmc[0], args.ingest_pmc[1], cfg.name + "+sampled",
                              (STREAM_KERNEL, "residual_segments_kernel"))
        return ingest_pmc(args.ingest_pmc[0], args.ingest_pmc[1], cfg.name)

    import numpy as np
    import torch

    from paper_2604_13634_amd import binding as csd

    from gen.device import to_device_logits

    torch.cuda.set_device(0)
    if args.path == "sampled":
        return bench_sampled(args, cfg)
    w = Workload(cfg)
    rows = cfg.rows
    n_ring = max(4, int(math.ceil(args.ring_bytes / cfg.bytes_per_step)))
    if args.graph:
        n_ring = min(n_ring, 64)
    if args.pmc_run:
        n_ring, args.steps, args.warmup = 4, 8, 2

    # ---- inputs: generated on the host, copied to HBM before anything is timed
    t_gen = time.perf_counter()
    ring_host, ring_z, ring_d = [], [], []
    for s in range(n_ring):
        z, d = w.step(s, threads=args.gen_threads)
        ring_z.append(to_device_logits(z))
        ring_d.append(torch.from_numpy(d).cuda())
        if s < 4:
            ring_host.append((z, d))
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen

    dt = csd.CSD_DTYPE_F32 if cfg.dtype == "f32" else csd.CSD_DTYPE_BF16
    bf = csd.VerifyBuffers.allocate(cfg.B, cfg.k, cfg.V, dt)

    def timed_steps(flags, steps, warmup):
        ocm = csd.new_ocm(cfg.capacity)
        for i in range(warmup):
            csd.csd_verify(ring_z[i % n_ring], ring_d[i % n_ring], cfg.tau, cfg.lam, ocm, flags, buffers=bf)
        if args.graph:                                # one captured step per ring slot, replayed in the timed loop
            torch.cuda.synchronize()
            graphs = []
            for j in range(n_ring):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    csd.csd_verify(ring_z[j], ring_d[j], cfg.tau, cfg.lam, ocm, flags, buffers=bf)
                graphs.append(g)
            csd.csd_ocm_reset(ocm)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            e0.record()
            for i in range(steps):
                graphs[(warmup + i) % n_ring].replay()
            e1.record()
            torch.cuda.synchronize()
            return time.perf_counter() - t0, ocm, e0.elapsed_time(e1) / steps
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()                                   # events on the stream the kernels are launched on
        for i in range(steps):
            j = (warmup + i) % n_ring
            csd.csd_verify(ring_z[j], ring_d[j], cfg.tau, cfg.lam, ocm, flags, buffers=bf)
        e1.record()
        torch.cuda.synchronize()
        return time.perf_counter() - t0, ocm, e0.elapsed_time(e1) / steps

    if args.pmc_run:
        timed_steps(csd.CSD_APPLY_UPDATES, args.steps, args.warmup)
        src = torch.empty(COPY_BYTES, dtype=torch.uint8, device="cuda")
        src.random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print("pmc-run done: %d csd_verify steps of %s, 3 copies of %d bytes" % (args.steps + args.warmup, cfg.name, COPY_BYTES))
        return 0

    # ---- the headline: whole hot path (two launches per step), memory updates applied
    elapsed, ocm, step_ms_events = timed_steps(csd.CSD_APPLY_UPDATES, args.steps, args.warmup)
    ms_per_step = elapsed / args.steps * 1e3
    value = rows * args.steps / elapsed
    accept_rate = float(bf.accept_len.float().mean().item()) / max(cfg.k, 1)
    status = bf.status.cpu().numpy().view(np.uint32).tolist()
    elapsed_noupd, _, _ = timed_steps(0, args.steps, args.warmup)

    # ---- for reference: two independent batches in flight (two streams, each with its own buffers and memory),
    # so that one batch's finish kernel overlaps the other's streaming pass
    def two_stream_rate(steps):
        sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
        lanes = []
        for st in (sa, sb):
            with torch.cuda.stream(st):
                lanes.append((st, csd.VerifyBuffers.allocate(cfg.B, cfg.k, cfg.V, dt), csd.new_ocm(cfg.capacity)))
        torch.cuda.synchronize()
        for i in range(4):
            for st, b2, o2 in lanes:
                with torch.cuda.stream(st):
                    csd.csd_verify(ring_z[i % n_ring], ring_d[i % n_ring], cfg.tau, cfg.lam, o2, buffers=b2)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            st, b2, o2 = lanes[i & 1]
            with torch.cuda.stream(st):
                csd.csd_verify(ring_z[i % n_ring], ring_d[i % n_ring], cfg.tau, cfg.lam, o2, buffers=b2)
        torch.cuda.synchronize()
        return rows * steps / (time.perf_counter() - t0)

    rate_two_streams = two_stream_rate(args.steps)

    # ---- the dominant kernel: the streaming pass (csd_row_partials launches exactly the kernel and grid that
    # csd_verify launches first), same ring, events on the launch stream
    part = csd.csd_row_partials(ring_z[0])
    for i in range(args.warmup):
        csd.csd_row_partials(ring_z[i % n_ring], part)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    ev0.record()
    for i in range(args.steps):
        csd.csd_row_partials(ring_z[(args.warmup + i) % n_ring], part)
    ev1.record()
    torch.cuda.synchronize()
    k_ms = ev0.elapsed_time(ev1) / args.steps
    alg_bytes = rows * cfg.V * cfg.itemsize            # every logit read once; partials and outputs are a few KB
    achieved = alg_bytes / (k_ms * 1e-3) / 1e9

    traffic = None
    if os.path.exists(TRAFFIC_FILE):
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f)
        ent = rec.get(cfg.name)
        if ent and ent.get("kernel_fingerprint") == kernel_fingerprint():
            traffic = ent["hbm_bytes_per_launch"]

    out = {
        "metric": "verified draft positions/sec + achieved HBM GB/s (% of peak) of csd_verify",
        "value": value,
        "unit": "positions/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": cfg.name, "B": cfg.B, "k": cfg.k, "V": cfg.V, "logits_storage": cfg.dtype,
            "positions_per_step": rows, "draft_positions_per_step": cfg.B * cfg.k,
            "tau": cfg.tau, "lambda": cfg.lam, "ocm_capacity": cfg.capacity, "ocm_updates": "applied",
            "launch": "graph replay" if args.graph else "two kernel launches per step",
            "ring_steps": n_ring, "ring_bytes": n_ring * cfg.bytes_per_step,
            "positions_per_s_without_ocm_updates": rows * args.steps / elapsed_noupd,
            "ms_per_step_without_ocm_updates": elapsed_noupd / args.steps * 1e3,
            "ms_per_step_by_stream_events": step_ms_events,
            "positions_per_s_two_batches_in_flight": rate_two_streams,
            "whole_path_GBps": alg_bytes / (ms_per_step * 1e-3) / 1e9,
            "whole_path_frac_of_hbm_peak": alg_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "accept_rate_last_step": accept_rate, "status_counters": status,
            "input_generation_s": t_gen,
        },
        "roofline": {
            "bound": "hbm", "kernel": "%s<%s>" % (STREAM_KERNEL, cfg.dtype), "achieved": achieved,
            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
            "kernel_ms": k_ms, "algorithmic_bytes_per_launch": alg_bytes,
        },
    }

    # ---- CPU baseline: the oracle as it stands, on the host cores, on a bounded sample of the same workload
    if not args.no_cpu_baseline:
        from oracle import csd_oracle as O
        cores = min(16, len(os.sched_getaffinity(0)))
        n_cpu_steps = len(ring_host)
        if cfg.bytes_per_step < (64 << 20):          # small workloads: regenerate more steps for a stable number
            extra = min(cfg.steps, max(4, int((256 << 20) // cfg.bytes_per_step)))
            ring_host = [w.step(s, threads=args.gen_threads) for s in range(extra)]
            n_cpu_steps = extra
        orc = O.CSDOracle(capacity=cfg.capacity)
        O.row_stats(ring_host[0][0][:1])             # load the library outside the timed part
        t0 = time.perf_counter()
        passes = 4 if cfg.bytes_per_step >= (64 << 20) else 1      # about 10-30 core-seconds in all
        for _ in range(passes):
            for z, d in ring_host:
                orc.verify_step(z, d, tau=np.float32(cfg.tau), lam=cfg.lam, threads=cores)
        n_cpu_steps *= passes
        t_cpu = time.perf_counter() - t0
        out["cpu_baseline"] = {
            "value": rows * n_cpu_steps / t_cpu, "unit": "positions/s", "cores": cores, "kind": "oracle",
            "sample": "%d steps of %s (%d positions), fp64 oracle, rows split over %d threads, scan and memory serial"
                      % (n_cpu_steps, cfg.name, rows * n_cpu_steps, cores),
            "seconds": t_cpu,
        }

    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
