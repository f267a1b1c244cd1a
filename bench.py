#!/usr/bin/env python3
"""Benchmark of the QESGD hot path on one MI355X.

A step is one synchronous round over one batch of synthetic input, already resident in HBM:
  1. qesgd_quantize_pack_batched   K simulated workers' vectors -> K packed blocks
  2. qesgd_unpack_aggregate_update K packed blocks + w_t, zsum  -> zbar, u, zsum
Reported: whole-step throughput in GB/s of algorithmic bytes (K*(4d+P) + K*P + 20d per step,
P = packed bytes per worker), per-phase GB/s and parameters/s, the roofline of the dominant
kernel from HIP events on the launch stream, and the CPU oracle timed on a bounded sample.
"""
import argparse
from dataclasses import replace
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E peak


def algorithmic_bytes(cfg, lay):
    P = lay.payload_bytes
    q = cfg.K * (4 * cfg.d + P)          # read K vectors, write K packed payloads
    uau = cfg.K * P + 20 * cfg.d         # read K payloads + w + zsum, write zbar + u + zsum
    return q, uau


def host_cpu():
    """Model name and online CPU count of the host the oracle is timed on."""
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return {"model": model, "online_cpus": os.cpu_count()}


class one_core:
    """Pins the calling thread to one host core for the timed part of the CPU baseline (the oracle
    is single-threaded; this keeps it from migrating), and restores the mask afterwards."""

    def __enter__(self):
        self.allowed, self.core = None, None
        try:
            self.allowed = os.sched_getaffinity(0)
            self.core = sorted(self.allowed)[len(self.allowed) // 2]
            os.sched_setaffinity(0, {self.core})
        except (AttributeError, OSError):
            self.allowed = None
        return self

    def __exit__(self, *exc):
        if self.allowed:
            os.sched_setaffinity(0, self.allowed)
        return False


def cpu_baseline(cfg, slab, w, lay, center=False, norm_kind=0, budget_elems=1 << 26):
    """The oracle as it stands, one host thread, on a bucket-aligned prefix of the same workload
    (the whole vector when the bucket is wider than the budget, or with budget_elems=None)."""
    import numpy as np
    from oracle import qesgd_oracle as oracle
    B = min(cfg.bucket, cfg.d)
    ds = cfg.d if budget_elems is None else min(cfg.d, max(B, (budget_elems // B) * B))
    host = slab[:, :ds].cpu().numpy()
    wh = w[:ds].cpu().numpy()
    with one_core() as pin:
        t0 = time.perf_counter()
        planes = [oracle.quantize_pack(host[k], cfg.s, cfg.bucket, cfg.seed, 0, k, center=wh if center else None,
                                       norm_kind=norm_kind) for k in range(cfg.K)]
        t1 = time.perf_counter()
        norms = np.stack([p[0] for p in planes])
        sw = np.stack([p[1] for p in planes])
        lw = np.stack([p[2] for p in planes])
        t2 = time.perf_counter()
        zbar = oracle.unpack_aggregate(norms, sw, lw, ds, cfg.s, cfg.bucket)
        oracle.apply_update(wh, zbar, np.zeros(ds, np.float32))
        t3 = time.perf_counter()
    pinned = pin.core
    nb, nsw, nlw, _, _ = oracle.shape(ds, cfg.s, cfg.bucket)
    P = 4 * (nb + nsw + nlw)
    qb, ub = cfg.K * (4 * ds + P) + (4 * ds if center else 0), cfg.K * P + 20 * ds
    tq, tu = t1 - t0, t3 - t2
    return {
        "value": round((qb + ub) / (tq + tu) / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": f"first {ds} of {cfg.d} coordinates of all {cfg.K} workers, one round "
                  f"({cfg.K * ds} coordinate quantisations)",
        "quantize_GBps": round(qb / tq / 1e9, 4), "aggregate_update_GBps": round(ub / tu / 1e9, 4),
        "quantize_params_per_s": round(cfg.K * ds / tq), "aggregate_update_params_per_s": round(ds / tu),
        "seconds": round(tq + tu, 2), "host": host_cpu(), "pinned_to_core": pinned,
    }


def quantize_kernels(cfg, args, workspace_bytes):
    """Names of the kernels one quantize-pack call launches for this shape (what rocprofv3 will list)."""
    B = min(cfg.bucket, cfg.d)
    if workspace_bytes:
        return "k_tile_partials(_fast) + k_finish_norms + k_quantize_pack_pre_fast (two passes, per group of workers)"
    pow2 = B & (B - 1) == 0
    m = cfg.s.bit_length() - 1
    if pow2 and B >= 32 and args.norm == "l2" and 32 % m == 0:
        return "k_quantize_pack_fast"
    return "k_quantize_pack"


def load_traffic(workload):
    """Measured HBM bytes per launch (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, calibrated on a
    copy), if a summary for this workload has been committed under profiles/."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.json")
    if os.path.exists(path):
        with open(path) as fh:
            return json.load(fh)
    return None


def copy_calibration(args, torch, dev):
    """--copy-calibration: one 1 GiB device-to-device copy, the reference point for --pmc byte counters."""
    if args.copy_calibration:
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b


def bench_fixed_grid(args, cfg, torch, B, synth, dev):
    """Server-to-worker direction with the quantiser as the paper writes it (Eq. (1)-(2), b = 8, the
    paper's setting): one step = qesgd_quantize_fixed of a d-vector + qesgd_dequantize_fixed_update
    (z, u = w + z, zsum += z)."""
    import numpy as np
    d, b = cfg.d, 8
    x = synth.worker_vector(cfg, 0, dev)
    w = synth.snapshot(cfg, dev)
    delta = float(np.float32(4.0 * float(x.std()) / 128.0))      # range = 4 standard deviations
    codes = torch.empty((d * b + 31) // 32, dtype=torch.int32, device=dev)
    z = torch.empty(d, device=dev)
    u = torch.empty(d, device=dev)
    zsum = torch.zeros(d, device=dev)
    stream = torch.cuda.current_stream()
    copy_calibration(args, torch, dev)
    variant = f"{cfg.name}_fixed_b{b}"
    traffic = load_traffic(variant) or {}

    def step(r, ev=None):
        if ev:
            ev[0].record(stream)
        B.qesgd_quantize_fixed(x, None, d, delta, b, cfg.seed, r, 0, codes, stream)
        if ev:
            ev[1].record(stream)
        B.qesgd_dequantize_fixed_update(codes, d, delta, b, w, z, u, zsum, stream)
        if ev:
            ev[2].record(stream)

    for r in range(args.warmup):
        step(r)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for r in range(args.steps):
        step(args.warmup + r, evs[r])
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / args.steps
    tq = sum(e[0].elapsed_time(e[1]) for e in evs) / len(evs)
    td = sum(e[1].elapsed_time(e[2]) for e in evs) / len(evs)
    cb = 4 * ((d * b + 31) // 32)
    qb, db = 4 * d + cb, cb + 20 * d                               # read x, write codes | read codes, w, zsum; write z, u, zsum
    out = {
        "metric": "fixed-grid quantize and dequantize+update GB/s (fp32 params) and % of HBM peak",
        "value": round((qb + db) / ms_step / 1e6, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{variant}: {cfg.name} shape, fixed grid: d={d} ({cfg.model}), b={b}, delta={delta:.3e}, "
                               f"entries {cfg.entries}, seed {cfg.seed}", "d": d, "b": b},
        "phases": {
            "quantize_fixed": {"algorithmic_bytes": qb, "ms_avg": round(tq, 4), "GBps": round(qb / tq / 1e6, 1),
                               "frac_of_hbm_peak": round(qb / tq / 1e6 / HBM_PEAK_GBPS, 4),
                               "params_per_s": round(d / tq * 1e3)},
            "dequantize_fixed_update": {"algorithmic_bytes": db, "ms_avg": round(td, 4),
                                        "GBps": round(db / td / 1e6, 1),
                                        "frac_of_hbm_peak": round(db / td / 1e6 / HBM_PEAK_GBPS, 4),
                                        "params_per_s": round(d / td * 1e3)}},
    }
    dom = "quantize_fixed" if tq >= td else "dequantize_fixed_update"
    out["roofline"] = {"kernel": "k_" + dom, "bound": "hbm", "achieved": out["phases"][dom]["GBps"],
                       "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": out["phases"][dom]["frac_of_hbm_peak"],
                       "traffic": traffic.get(dom)}
    if not args.no_cpu_baseline:
        from oracle import qesgd_oracle as oracle
        ds = min(d, 1 << 26)
        xh, wh = x[:ds].cpu().numpy(), w[:ds].cpu().numpy()
        with one_core():
            t0 = time.perf_counter()
            oc = oracle.quantize_fixed(xh, delta, b, cfg.seed, 0, 0)
            t1 = time.perf_counter()
            oracle.dequantize_fixed_update(oc, ds, delta, b, w_snap=wh, zsum=np.zeros(ds, np.float32))
            t2 = time.perf_counter()
        sb = 4 * ds + ds + ds + 20 * ds
        out["cpu_baseline"] = {"value": round(sb / (t2 - t0) / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
                               "sample": f"first {ds} of {d} coordinates, one step",
                               "quantize_params_per_s": round(ds / (t1 - t0)),
                               "dequantize_update_params_per_s": round(ds / (t2 - t1)),
                               "seconds": round(t2 - t0, 2), "host": host_cpu()}
    print(json.dumps(out), flush=True)


PROBE_READ, PROBE_COPY, PROBE_QUANTIZE_MIX, PROBE_UPDATE_MIX, PROBE_BYTE_CODES_MIX = range(5)


def load_probe():
    """The plain streaming kernels of libqesgd_bench_probe.so (a benchmark aid built next to the
    library, not part of its ABI).  Returns probe(pattern, a, b, c, d, e, n, torch_stream)."""
    import ctypes as C
    path = os.path.join(ROOT, "paper_1901_03040_amd", "libqesgd_bench_probe.so")
    if not os.path.exists(path):
        raise RuntimeError(f"{path} not found: build it with `python -m paper_1901_03040_amd.build`")
    L = C.CDLL(path)
    L.qesgd_bench_probe.argtypes = [C.c_uint32] + [C.c_void_p] * 5 + [C.c_uint64, C.c_void_p]
    L.qesgd_bench_probe.restype = C.c_int

    def probe(pattern, a, b, c, d, e, n, stream):
        ptr = [None if t is None else C.c_void_p(t.data_ptr()) for t in (a, b, c, d, e)]
        rc = L.qesgd_bench_probe(int(pattern), *ptr, int(n), C.c_void_p(stream.cuda_stream))
        if rc != 0:
            raise RuntimeError(f"qesgd_bench_probe({pattern}) failed with code {rc}")
    return probe


def bench_ceilings(args, cfg, torch, B, synth, dev):
    """Plain streaming kernels with the two hot kernels' access mixes, on the workload's footprint:
    what this machine reaches with no arithmetic.  Prints one JSON line of its own."""
    stride = synth.slab_stride(cfg.d)
    n_slab = cfg.K * stride // 4096 * 4096            # floats the quantiser reads per round
    n_vec = cfg.d // 4096 * 4096                      # floats per parameter-sized vector
    slab = synth.worker_slab(cfg, dev).view(-1)
    planes = [torch.empty(n_slab // 32, dtype=torch.float32, device=dev) for _ in range(2)]
    vec = [torch.empty(n_vec, dtype=torch.float32, device=dev).normal_() for _ in range(5)]
    stream = torch.cuda.current_stream()
    n_copy = n_slab
    dst = torch.empty(n_copy, dtype=torch.float32, device=dev)
    probe = load_probe()
    cases = [
        ("read_only", PROBE_READ, (slab, dst, None, None, None), n_slab, 4 * n_slab),
        ("copy", PROBE_COPY, (slab, dst, None, None, None), n_copy, 8 * n_copy),
        ("quantize_mix_read_plus_2_packed_planes", PROBE_QUANTIZE_MIX, (slab, planes[0], planes[1], None, None),
         n_slab, 4 * n_slab + 2 * (n_slab // 8)),
        ("byte_codes_mix_read_plus_1_byte_per_float", PROBE_BYTE_CODES_MIX, (vec[0], vec[1], None, None, None),
         n_vec, 5 * n_vec),
        ("update_mix_2_reads_3_writes", PROBE_UPDATE_MIX, tuple(vec), n_vec, 20 * n_vec),
    ]
    out = {"ceilings": {}, "unit": "GB/s", "config": {"workload": f"{cfg.name} footprint: d={cfg.d}, K={cfg.K}"}, "steps": args.steps,
           "warmup": args.warmup, "hbm_peak": HBM_PEAK_GBPS}
    for name, pattern, bufs, n, nbytes in cases:
        ms = []
        for r in range(args.warmup + args.steps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            probe(pattern, *bufs, n, stream)
            e1.record(stream)
            e1.synchronize()
            if r >= args.warmup:
                ms.append(e0.elapsed_time(e1))
        ms.sort()
        med = ms[len(ms) // 2]
        out["ceilings"][name] = {"bytes": nbytes, "ms_median": round(med, 4), "ms_min": round(ms[0], 4),
                                 "GBps": round(nbytes / med / 1e6, 1),
                                 "frac_of_hbm_peak": round(nbytes / med / 1e6 / HBM_PEAK_GBPS, 4)}
    if args.sweeps:
        # Back-to-back read sweeps over buffers of growing size: what a re-read gains when the
        # buffer still sits in the 256 MB memory-side cache (it does below that size).
        out["resident_sweeps"] = {}
        for mib in (32, 64, 128, 200, 256, 512, 1024, 4096):
            n = mib * (1 << 20) // 4
            a = torch.empty(n, dtype=torch.float32, device=dev).normal_()
            sink = torch.empty(n, dtype=torch.float32, device=dev)       # never written for ordinary data
            for _ in range(3):
                probe(PROBE_READ, a, sink, None, None, None, n, stream)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(20):
                probe(PROBE_READ, a, sink, None, None, None, n, stream)
            e1.record(stream)
            e1.synchronize()
            ms = e0.elapsed_time(e1) / 20
            out["resident_sweeps"][f"{mib}MiB"] = {"us_per_sweep": round(ms * 1e3, 1), "GBps": round(4 * n / ms / 1e6, 1)}
            del a, sink
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="cfg5", help="cfg1..cfg5 (default: the largest, VGG-16-sized)")
    ap.add_argument("--bucket", default=None,
                    help="override the configuration's bucket size: a number (a multiple of 32), or 'whole' "
                         "for one scale over the whole vector (the two-pass path of wide buckets)")
    ap.add_argument("--s", type=int, default=None, help="override the configuration's number of levels")
    ap.add_argument("--norm", default="l2", choices=["l2", "max"], help="bucket scale: L2 norm (default) or max |v|")
    ap.add_argument("--center", action="store_true",
                    help="the workers hold x_k = w_t + z_k and the quantiser forms x_k - w_t itself (reads 8 B per coordinate)")
    ap.add_argument("--path", default="qesgd", choices=["qesgd", "fixed"],
                    help="qesgd: bucketed quantize-pack + unpack-aggregate-update (the headline path); "
                         "fixed: the paper-literal fixed-grid quantiser (b = 8) + its fused inverse")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step replayed from a HIP graph (adds graph_replay_ms_per_step)")
    ap.add_argument("--one-call", action="store_true",
                    help="also time the step through qesgd_round (a whole round in one call / one launch; adds one_call)")
    ap.add_argument("--ceilings", action="store_true",
                    help="instead of the benchmark, time plain streaming kernels with the hot kernels' "
                         "access mixes on the workload's footprint (practical HBM ceilings of this machine)")
    ap.add_argument("--sweeps", action="store_true",
                    help="with --ceilings: also time 20 back-to-back read sweeps over buffers of 32 MiB .. 4 GiB "
                         "(reach of the memory-side cache)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-full", action="store_true",
                    help="time the CPU oracle on the whole workload instead of a 2^26-coordinate prefix "
                         "(cfg5: about 25 s)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 1 GiB device copy (reference point for --pmc byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (K workers are K device buffers); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1901_03040_amd import binding as B
    from paper_1901_03040_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    dev = "cuda:0"
    cfg = synth.by_name(args.config)
    variant = cfg.name
    if args.bucket is not None:
        bucket = cfg.d if args.bucket == "whole" else int(args.bucket)
        cfg = replace(cfg, bucket=bucket)
        variant += "_whole" if bucket >= cfg.d else f"_b{bucket}"
    if args.s is not None:
        cfg = replace(cfg, s=args.s)
        variant += f"_s{args.s}"
    if args.norm == "max":
        variant += "_max"
    if args.center:
        variant += "_center"
    if args.ceilings:
        return bench_ceilings(args, cfg, torch, B, synth, dev)
    if args.path == "fixed":
        return bench_fixed_grid(args, cfg, torch, B, synth, dev)
    lay = B.qesgd_layout_query(cfg.d, cfg.s, cfg.bucket)
    slab = synth.worker_slab(cfg, dev)
    w = synth.snapshot(cfg, dev)
    center = None
    if args.center:
        slab[:, :cfg.d] += w          # x_k = w_t + z_k; the kernel quantises fl(x_k - w_t)
        center = w
    norm_kind = B.NORM_MAX if args.norm == "max" else B.NORM_L2
    packed = B.alloc_packed(lay, cfg.K, dev)
    zbar = torch.empty(cfg.d, device=dev)
    u = torch.empty(cfg.d, device=dev)
    zsum = torch.zeros(cfg.d, device=dev)
    wsb = B.qesgd_workspace_bytes(cfg.d, cfg.s, cfg.bucket, cfg.K)
    ws = torch.empty(max(wsb // 4, 1), dtype=torch.float32, device=dev) if wsb else None
    stream = torch.cuda.current_stream()

    copy_calibration(args, torch, dev)

    def step(r, events=None):
        if events is not None:
            events[0].record(stream)
        B.qesgd_quantize_pack_batched(slab, slab.stride(0), center, cfg.d, cfg.s, cfg.bucket, norm_kind,
                                      cfg.seed, r, cfg.K, packed, packed.stride(0), ws, stream)
        if events is not None:
            events[1].record(stream)
        B.qesgd_unpack_aggregate_update(packed, packed.stride(0), cfg.K, cfg.d, cfg.s, cfg.bucket, w, zbar, u,
                                        zsum, stream)
        if events is not None:
            events[2].record(stream)

    for r in range(args.warmup):
        step(r)
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for r in range(args.steps):
        step(args.warmup + r, evs[r])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_step = (t1 - t0) * 1e3 / args.steps
    tq = sorted(e[0].elapsed_time(e[1]) for e in evs)
    tu = sorted(e[1].elapsed_time(e[2]) for e in evs)
    tq_avg, tu_avg = sum(tq) / len(tq), sum(tu) / len(tu)
    qb, ub = algorithmic_bytes(cfg, lay)
    if args.center:
        qb += 4 * cfg.d               # w_t is shared by the K workers of one GPU: read once
    traffic = load_traffic(variant) or {}

    def phase(bytes_, ms_avg, ms_sorted, params):
        return {"algorithmic_bytes": bytes_, "ms_avg": round(ms_avg, 4), "ms_median": round(ms_sorted[len(ms_sorted) // 2], 4),
                "ms_min": round(ms_sorted[0], 4), "GBps": round(bytes_ / ms_avg / 1e6, 1),
                "frac_of_hbm_peak": round(bytes_ / ms_avg / 1e6 / HBM_PEAK_GBPS, 4),
                "params_per_s": round(params / ms_avg * 1e3)}

    phases = {"quantize_pack": phase(qb, tq_avg, tq, cfg.K * cfg.d),
              "unpack_aggregate_update": phase(ub, tu_avg, tu, cfg.d)}
    dom = "quantize_pack" if tq_avg >= tu_avg else "unpack_aggregate_update"

    def roofline(name):
        ph = phases[name]
        launches = {"quantize_pack": quantize_kernels(cfg, args, wsb),
                    "unpack_aggregate_update": "k_unpack_aggregate_update"}[name]
        return {"kernel": launches, "bound": "hbm", "achieved": ph["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": ph["frac_of_hbm_peak"], "traffic": traffic.get(name)}

    out = {
        "metric": "quantize+pack and unpack+aggregate+update GB/s (fp32 params) and % of HBM peak",
        "value": round((qb + ub) / ms_step / 1e6, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{variant}: d={cfg.d} ({cfg.model}), K={cfg.K}, s={cfg.s}, bucket={cfg.bucket}, "
                               f"norm {args.norm}, {'x - w_t formed in the kernel, ' if args.center else ''}"
                               f"entries {cfg.entries}, seed {cfg.seed}",
                   "d": cfg.d, "K": cfg.K, "s": cfg.s, "bucket": cfg.bucket, "norm": args.norm,
                   "center": bool(args.center),
                   "packed_bytes_per_worker": lay.payload_bytes},
        "frac_of_hbm_peak": round((qb + ub) / ms_step / 1e6 / HBM_PEAK_GBPS, 4),
        "params_per_s": round(cfg.K * cfg.d / ms_step * 1e3),
        "phases": phases,
        "roofline": roofline(dom),
        "roofline_other": roofline("unpack_aggregate_update" if dom == "quantize_pack" else "quantize_pack"),
    }
    if args.graph:
        # The same step replayed from a HIP graph (launch-bound shapes: cfg1, cfg2).  The round
        # argument is frozen at capture, so every replay draws the same variates.
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            B.qesgd_quantize_pack_batched(slab, slab.stride(0), center, cfg.d, cfg.s, cfg.bucket, norm_kind,
                                          cfg.seed, 0, cfg.K, packed, packed.stride(0), ws)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            B.qesgd_quantize_pack_batched(slab, slab.stride(0), center, cfg.d, cfg.s, cfg.bucket, norm_kind,
                                          cfg.seed, 0, cfg.K, packed, packed.stride(0), ws)
            B.qesgd_unpack_aggregate_update(packed, packed.stride(0), cfg.K, cfg.d, cfg.s, cfg.bucket, w, zbar, u,
                                            zsum)
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        out["graph_replay_ms_per_step"] = round((time.perf_counter() - g0) * 1e3 / args.steps, 4)
    if args.one_call:
        # The same step through qesgd_round: one launch where the shape allows it (it writes the
        # packed blocks but does not read them back: K*P bytes fewer than the two-call form).
        def round_call(r):
            B.qesgd_round(slab, slab.stride(0), center, cfg.d, cfg.s, cfg.bucket, norm_kind, cfg.seed, r, cfg.K,
                          packed, packed.stride(0), w, zbar, u, zsum, workspace=ws, stream=stream)
        for r in range(args.warmup):
            round_call(r)
        torch.cuda.synchronize()
        o0 = time.perf_counter()
        for r in range(args.steps):
            round_call(args.warmup + r)
        torch.cuda.synchronize()
        oms = (time.perf_counter() - o0) * 1e3 / args.steps
        moved = qb + ub - cfg.K * lay.payload_bytes
        out["one_call"] = {"ms_per_step": round(oms, 4), "bytes_moved": moved,
                           "GBps_of_bytes_moved": round(moved / oms / 1e6, 1),
                           "GBps_by_the_two_call_accounting": round((qb + ub) / oms / 1e6, 1)}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, slab, w, lay, center=args.center, norm_kind=norm_kind,
                                           budget_elems=None if args.cpu_full else 1 << 26)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
