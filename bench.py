#!/usr/bin/env python3
"""Benchmark of the compress/decompress hot path on one MI355X.

A step is one pass of the per-iteration path over one batch: error-bound controller ->
compress -> decompress of the workload-3 payload (one rank's all-to-all share: 128 tables x
8192 lookups x dim 128 fp32 = 512 MiB, synthetic, resident in HBM before the timed region).
The statistics reduction is offline in the paper (Section III-A) and is timed separately.

Prints ONE JSON line (see the keys below).  `value` = uncompressed payload bytes that went
through compress AND decompress per second of step time.
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

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth
TARGET_FRAC = 0.60      # what each direction is asked to reach on the 512 MiB workload
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "cfg3_hbm_traffic_pmc.txt")
ORACLE_SAMPLE_BYTES = 64 << 20  # the oracle checks a workload's first tables, this many bytes of them at most


def profiled_traffic():
    """HBM bytes per launch by kernel name, from the committed summary of the FETCH_SIZE / WRITE_SIZE counter runs (the
    counters cannot be collected from inside this process).  Its line `bytes per launch: k_x 1.2e6, k_y ...` is what
    is read; no such file or line, or a kernel it does not name: no figure."""
    try:
        with open(TRAFFIC_PROFILE) as f:
            for line in f:
                if line.startswith("bytes per launch:"):
                    items = [it.split() for it in line.split(":", 1)[1].strip().rstrip(".").split(",")]
                    return {name: float(val) for name, val in items}
    except (OSError, ValueError):
        pass
    return {}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg3", choices=["cfg3", "cfg3-small"])
    ap.add_argument("--chunk-symbols", type=int, default=256)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-level", type=int, default=1)
    ap.add_argument("--carry-codebook", action="store_true",
                    help="time the single-pass path (DLC_FLAG_CARRY_CODEBOOK: each step is coded with the codebook built "
                         "from the previous step's payload) instead of the default two-pass path")
    ap.add_argument("--sample-codebook", action="store_true",
                    help="time the single-pass path that builds every table's codebook from a sample of the step's own "
                         "payload (DLC_FLAG_SAMPLE_CODEBOOK) instead of the default two-pass path")
    ap.add_argument("--row-match", action="store_true",
                    help="time the path with the vector-based LZ step on every table (DLC_FLAG_ROW_MATCH) instead of the "
                         "default path; the roofline object then still prices the kernel the profile slots see")
    ap.add_argument("--no-workloads", action="store_true",
                    help="leave out the 'workloads' list (the five synthetic workloads, each timed both ways and checked "
                         "against the oracle on its first tables)")
    ap.add_argument("--all-workloads", action="store_true",
                    help="the long form of the 'workloads' list: the oracle over every whole payload, workload 3 split over "
                         "8 and 32 destinations and with row matching, workload 5 as a run of 200 iterations (about a "
                         "minute more)")
    ap.add_argument("--copy-reference", action="store_true",
                    help="also run three plain device copies of the payload (the known-size kernel that HBM counters are scaled by)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import dlc_workloads as W
    from paper_2407_04272_amd import binding as b

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.workload == "cfg3":
        w = W.workload3(device=dev)
    else:
        w = W.workload3(T=16, B=8192, D=128, rows=20000, device=dev)
    d = w.payload
    T, B, D = d.shape
    payload_bytes = d.numel() * 4
    if args.carry_codebook + args.row_match + args.sample_codebook > 1:
        print("bench.py: --carry-codebook, --sample-codebook and --row-match are different paths; pick one", file=sys.stderr)
        sys.exit(2)
    flags = (b.FLAG_CARRY_CODEBOOK if args.carry_codebook else b.FLAG_SAMPLE_CODEBOOK if args.sample_codebook
             else b.FLAG_ROW_MATCH if args.row_match else 0)
    ctx = b.Context(b.make_config(b.F32, T, B, D, chunk_symbols=args.chunk_symbols, flags=flags))

    # offline analysis (Section III-A): statistics -> table classes; timed on its own
    probe_first = np.full(T, 1e-3, np.float32)
    st0 = ctx.stats(d, probe_first)
    probe = np.array([0.03 * (s.max - s.min) for s in st0], np.float32)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    st = ctx.stats(d, probe)
    stats_ms = (time.perf_counter() - t0) * 1e3
    p = b.ControllerParams(mode=1, decay_kind=b.DECAY_STEPWISE, global_eb=w.meta["global_eb"], alpha=w.meta["alpha"],
                           beta=w.meta["beta"], h_large=0.0, h_small=0.05, decay_start=0, decay_len=100,
                           decay_steps=5, reserved=0, decay_mult0=2.0, eb_min=0.0, eb_max=0.0, rel_floor=0.0)
    # table-wise bounds only (workload 3): iteration past the decay phase
    it_fixed = 1000
    out = torch.zeros(payload_bytes, dtype=torch.uint8, device=dev)  # ample: the container is ~1/10 of this
    sizes = torch.zeros(1 + T, dtype=torch.int64, device=dev)
    rec = torch.empty_like(d)

    def step(i):
        ctx.set_error_bounds(stats=st, params=p, iteration=it_fixed)
        rc = ctx.compress(d, out, sizes)
        assert rc == 0, rc
        # the container size is known to the caller only after the size word came back; a real
        # pipeline gets it from the metadata exchange -- here the capacity stands in for it
        rc = ctx.decompress(out, out.numel(), rec)
        assert rc == 0, rc

    if args.copy_reference:
        for _ in range(3):
            rec.copy_(d)
        torch.cuda.synchronize()
    for i in range(args.warmup):
        step(i)
    assert ctx.sync_status() == 0
    total = int(sizes[0].item())
    assert total > 0
    cr = payload_bytes / total

    # every kernel once, outside the timed region (events around all of them would stretch the step by ~40 us)
    ctx.profile_enable(2)
    for i in range(max(3, args.warmup)):
        step(i)
    prof_all = ctx.profile_read()
    # the timed region: events around the dominant kernel of each direction only
    ctx.profile_enable(args.profile_level)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = ctx.profile_read()
    ctx.profile_enable(0)
    assert ctx.sync_status() == 0
    ms_per_step = dt / args.steps * 1e3
    value = payload_bytes / (dt / args.steps) / 1e9

    # each direction on its own (events on the stream the library launches on)
    def timed(fn, n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / n

    n_dir = max(5, args.steps // 2)
    comp_ms = timed(lambda: ctx.compress(d, out, sizes), n_dir)
    dec_ms = timed(lambda: ctx.decompress(out, total, rec), n_dir)
    assert ctx.sync_status() == 0

    # the bound holds on a sample of the output (the parity tests check everything element by element)
    ebs, _ = ctx.set_error_bounds(stats=st, params=p, iteration=it_fixed)
    idx = torch.randint(0, B * D, (4096,), device=dev)
    err = (d.view(T, -1)[:, idx].double() - rec.view(T, -1)[:, idx].double()).abs().amax(1).cpu().numpy()
    assert np.all(err <= ebs.astype(np.float64) * (1 + 1e-6)), "error bound violated"

    algo_bytes = payload_bytes * (1.0 + 1.0 / cr)  # read s + write s/CR per element (and the reverse)
    kern = {k: (ms / n if n else 0.0) for k, (ms, n) in prof.items()}          # timed region
    kern_all = {k: (ms / n if n else 0.0) for k, (ms, n) in prof_all.items()}  # pre-pass, every kernel
    # dominant kernel = the one with the largest average duration; its duration comes from the timed region when it is
    # one of the kernels timed there (the dominant kernel of a direction is), else from the pre-pass
    timed_kernels = [k for k in kern_all if kern_all[k] > 0]
    if timed_kernels:
        dom = max(timed_kernels, key=lambda k: kern_all[k])
        dom_ms = kern[dom] if kern.get(dom, 0) > 0 else kern_all[dom]
    else:
        dom, dom_ms = "dlc_compress (all kernels)", comp_ms
    # priced with the path's algorithmic bytes per element, s(1 + 1/CR), times the elements a launch processes (all of
    # them, for every streaming kernel here); the direction-level fractions are in compress_/decompress_roofline_frac
    dom_bytes = algo_bytes
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    # HBM bytes per launch of the dominant kernel, from the committed counter summary; it covers this workload only
    traffic = profiled_traffic().get(dom) if (args.workload == "cfg3" and args.chunk_symbols == 256 and not args.row_match) else None
    comp_frac = algo_bytes / (comp_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS
    dec_frac = algo_bytes / (dec_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS
    result = {
        "metric": "compress+decompress round-trip GB/s of uncompressed fp32 payload, 1 MI355X",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {T} tables x {B} lookups x dim {D} fp32 ({payload_bytes >> 20} MiB), "
                               "Zipf(1.05) single-hot, N(0,sigma_t), table-wise range-relative bounds 0.03",
                   "chunk_symbols": args.chunk_symbols, "radius": 512, "max_code_len": 12,
                   "codebook": ("carried from the previous step" if args.carry_codebook else
                                "built from a sample of the step's own payload" if args.sample_codebook else
                                "built from the step's own payload"),
                   "row_matching": bool(args.row_match)},
        "compression_ratio": round(cr, 3),
        "compress_GBps": round(payload_bytes / comp_ms / 1e6, 2), "compress_ms": round(comp_ms, 4),
        "decompress_GBps": round(payload_bytes / dec_ms / 1e6, 2), "decompress_ms": round(dec_ms, 4),
        "compress_roofline_frac": round(comp_frac, 4),
        "decompress_roofline_frac": round(dec_frac, 4),
        "stats_ms": round(stats_ms, 3), "stats_GBps": round(payload_bytes / stats_ms / 1e6, 2),
        "kernel_ms": {k: round(v, 4) for k, v in kern.items() if v > 0},
        "kernel_ms_all": {k: round(v, 4) for k, v in kern_all.items() if v > 0},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     # what the target is stated on: a whole call of each direction (all its kernels), same bytes
                     "direction_frac": {"compress": round(comp_frac, 4), "decompress": round(dec_frac, 4)},
                     "target_frac": TARGET_FRAC,
                     "target_met": {"compress": bool(comp_frac >= TARGET_FRAC), "decompress": bool(dec_frac >= TARGET_FRAC)}},
    }

    if not args.carry_codebook and not args.row_match and not args.sample_codebook:
        # for information: the same workload through the two single-pass paths (not part of `value`)
        for name, fl, note in (("carried_codebook", b.FLAG_CARRY_CODEBOOK,
                                "each call coded with the codebook of the previous call's payload (here the same "
                                "payload); see --carry-codebook"),
                               ("sampled_codebook", b.FLAG_SAMPLE_CODEBOOK,
                                "each call coded with the codebook of a sample of its own payload (four groups of "
                                "16384 elements per table); see --sample-codebook")):
            ctx2 = b.Context(b.make_config(b.F32, T, B, D, chunk_symbols=args.chunk_symbols, flags=fl))
            ctx2.set_error_bounds(eb=ebs)
            for _ in range(3):
                ctx2.compress(d, out, sizes)
            assert ctx2.sync_status() == 0
            total2 = int(sizes[0].item())
            comp2_ms = timed(lambda: ctx2.compress(d, out, sizes), n_dir)

            def step2():
                ctx2.compress(d, out, sizes)
                ctx2.decompress(out, out.numel(), rec)
            rt2_ms = timed(step2, n_dir)
            assert ctx2.sync_status() == 0
            algo2 = payload_bytes * (1.0 + total2 / payload_bytes)
            frac2 = algo2 / (comp2_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS
            result["roofline"]["direction_frac"]["compress_" + name] = round(frac2, 4)
            result["roofline"]["target_met"]["compress_" + name] = bool(frac2 >= TARGET_FRAC)
            result[name] = {"compress_ms": round(comp2_ms, 4),
                            "compress_GBps": round(payload_bytes / comp2_ms / 1e6, 2),
                            "compress_roofline_frac": round(frac2, 4),
                            "round_trip_GBps": round(payload_bytes / rt2_ms / 1e6, 2),
                            "compression_ratio": round(payload_bytes / total2, 3),
                            "note": note}
            del ctx2
        # leave the default path's container in `out` for the comparison below
        ctx.compress(d, out, sizes)
        assert ctx.sync_status() == 0

    if not args.no_cpu_baseline:
        import oracle
        x = d.cpu().numpy()
        carry = None
        if args.carry_codebook:  # the steady state of the chain: the counts of the same payload
            carry = oracle.compress(x, ebs, want_hist=True).hist
        t0 = time.perf_counter()
        o = oracle.compress(x, ebs, carry_hist=carry, row_match=(True if args.row_match else None),
                            sample_codebook=bool(args.sample_codebook))
        tc = time.perf_counter() - t0
        t0 = time.perf_counter()
        rc, orec = oracle.decompress(o.data, x.shape, np.float32)
        td = time.perf_counter() - t0
        assert o.rc == 0 and rc == 0
        same = bool(o.data.size == total and np.array_equal(o.data, out[:total].cpu().numpy()))
        result["cpu_baseline"] = {"value": round(payload_bytes / (tc + td) / 1e9, 4), "unit": "GB/s", "cores": 1,
                                  "kind": "oracle", "sample": "the full payload of the same workload, one pass",
                                  "compress_GBps": round(payload_bytes / tc / 1e9, 4),
                                  "decompress_GBps": round(payload_bytes / td / 1e9, 4),
                                  "container_identical_to_gpu": same}
    if args.all_workloads or not args.no_workloads:
        del d, rec, out
        torch.cuda.empty_cache()
        result["workloads"] = all_workloads(b, torch, np, W, dev, args.chunk_symbols, not args.no_cpu_baseline,
                                            long_form=args.all_workloads)
    print(json.dumps(result))


def _measure(b, torch, np, name, d, ebs, S, with_oracle, sample_bytes=None):
    """compress / decompress of one payload at the given bounds: both paths on the GPU, the oracle beside them (on the
    whole payload, or on its first tables up to sample_bytes: the library then compresses those tables on their own
    and the two containers are compared byte for byte)."""
    T, B, D = d.shape
    f16 = d.dtype == torch.float16
    nbytes = d.numel() * d.element_size()
    out = torch.zeros(max(nbytes, 1 << 20), dtype=torch.uint8, device=d.device)
    sizes = torch.zeros(1 + T, dtype=torch.int64, device=d.device)
    rec = torch.empty_like(d)
    row = {"workload": name, "shape": [T, B, D], "dtype": "f16" if f16 else "f32", "payload_MiB": round(nbytes / 2 ** 20, 3)}

    def timed(fn, n=20):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(3):
            fn()
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / n

    for key, flags in (("", 0), ("carried_", b.FLAG_CARRY_CODEBOOK), ("sampled_", b.FLAG_SAMPLE_CODEBOOK)):
        ctx = b.Context(b.make_config(b.F16 if f16 else b.F32, T, B, D, chunk_symbols=S, flags=flags))
        ctx.set_error_bounds(eb=ebs)
        c_ms = timed(lambda: ctx.compress(d, out, sizes))
        assert ctx.sync_status() == 0
        total = int(sizes[0].item())
        cr = nbytes / total
        algo = nbytes * (1.0 + 1.0 / cr)
        row[key + "compression_ratio"] = round(cr, 3)
        row[key + "compress_GBps"] = round(nbytes / c_ms / 1e6, 2)
        row[key + "compress_ms"] = round(c_ms, 4)
        row[key + "compress_roofline_frac"] = round(algo / (c_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)
        if not key:
            d_ms = timed(lambda: ctx.decompress(out, total, rec))
            assert ctx.sync_status() == 0
            row["decompress_GBps"] = round(nbytes / d_ms / 1e6, 2)
            row["decompress_ms"] = round(d_ms, 4)
            row["decompress_roofline_frac"] = round(algo / (d_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)
            eb_t = torch.from_numpy(np.asarray(ebs, np.float64)).to(d.device).view(T, 1, 1)
            fin = torch.isfinite(d)
            err = torch.where(fin, (d.double() - rec.double()).abs(), torch.zeros((), dtype=torch.float64, device=d.device))
            row["bound_held"] = bool((err <= eb_t * (1 + 1e-6)).all())
            data = out[:total].cpu().numpy()
        del ctx
    if with_oracle:
        import oracle
        Ts = T if sample_bytes is None else max(1, min(T, sample_bytes // (nbytes // T)))
        if Ts < T:  # the first Ts tables as a payload of their own, through the library again
            ctx = b.Context(b.make_config(b.F16 if f16 else b.F32, Ts, B, D, chunk_symbols=S))
            ctx.set_error_bounds(eb=ebs[:Ts])
            assert ctx.compress(d[:Ts], out, sizes[:1 + Ts]) == 0 and ctx.sync_status() == 0
            data = out[:int(sizes[0].item())].cpu().numpy()
            del ctx
        x = d[:Ts].cpu().numpy()
        t0 = time.perf_counter()
        o = oracle.compress(x, ebs[:Ts], S=S)
        tc = time.perf_counter() - t0
        t0 = time.perf_counter()
        rc, orec = oracle.decompress(o.data, x.shape, x.dtype)
        td = time.perf_counter() - t0
        u = np.uint16 if f16 else np.uint32
        row["oracle_GBps"] = round(x.nbytes / (tc + td) / 1e9, 4)
        row["oracle_sample"] = "the whole payload" if Ts == T else f"the first {Ts} of {T} tables"
        row["same_bytes_as_oracle"] = bool(o.rc == 0 and rc == 0 and o.data.size == data.size and np.array_equal(o.data, data)
                                           and np.array_equal(orec.view(u), rec[:Ts].cpu().numpy().view(u)))
    return row


def _measure_split(b, torch, np, d, ebs, S, n, with_oracle):
    """Workload 3 cut along the batch axis into n pieces (one per receiving GPU): one compress call writes n containers
    at fixed displacements; the receiver's side is n decompress calls, one per container."""
    T, B, D = d.shape
    Bp = B // n
    x = d.view(T, n, Bp, D).permute(1, 0, 2, 3).contiguous()          # [n][T][B/n][D]: the send buffer's layout
    nbytes = x.numel() * 4
    row = {"workload": f"3 split over {n} destinations ({T} x {Bp} x {D} each)", "payload_MiB": round(nbytes / 2 ** 20, 3)}
    out = torch.zeros(nbytes, dtype=torch.uint8, device=d.device)
    sizes = torch.zeros(1 + n * T + n, dtype=torch.int64, device=d.device)
    rec = torch.empty((T, Bp, D), dtype=torch.float32, device=d.device)
    stride = (out.numel() // n) & ~255

    def timed(fn, reps=20):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(3):
            fn()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / reps

    for key, flags in (("", 0), ("carried_", b.FLAG_CARRY_CODEBOOK)):
        ctx = b.Context(b.make_config(b.F32, T, Bp, D, chunk_symbols=S, flags=flags, num_dest=n))
        ctx.set_error_bounds(eb=ebs)
        c_ms = timed(lambda: ctx.compress(x, out, sizes))
        assert ctx.sync_status() == 0
        total = int(sizes[0].item())
        row[key + "compression_ratio"] = round(nbytes / total, 3)
        row[key + "compress_GBps"] = round(nbytes / c_ms / 1e6, 2)
        if not key:
            dsz = sizes[1 + n * T:].cpu().numpy()
            rec_all = torch.empty_like(x)
            d_ms = timed(lambda: ctx.decompress(out, out.numel(), rec_all))      # all containers, one call
            assert ctx.sync_status() == 0
            row["decompress_GBps"] = round(nbytes / d_ms / 1e6, 2)
            dctx = b.Context(b.make_config(b.F32, T, Bp, D, chunk_symbols=S))

            def dec_all():
                for k in range(n):
                    dctx.decompress(out[k * stride:], int(dsz[k]), rec)
            d_ms = timed(dec_all, 10)
            assert dctx.sync_status() == 0
            row["decompress_GBps_one_call_per_container"] = round(nbytes / d_ms / 1e6, 2)
            assert bool((rec_all[n - 1] == rec).all())
            eb_t = torch.from_numpy(np.asarray(ebs, np.float64)).to(d.device).view(T, 1, 1)
            row["bound_held"] = bool(((x[n - 1].double() - rec.double()).abs() <= eb_t * (1 + 1e-6)).all())
            if with_oracle:
                import oracle
                same = True
                for k in (0, n - 1):       # two pieces against the oracle (the parity tests compare every piece)
                    o = oracle.compress(x[k].cpu().numpy(), ebs, S=S)
                    got = out[k * stride:k * stride + int(dsz[k])].cpu().numpy()
                    same = same and o.rc == 0 and o.data.size == got.size and bool(np.array_equal(o.data, got))
                row["containers_identical_to_oracle"] = same
        del ctx
    return row


def _measure_rows(b, torch, np, d, ebs, S, with_oracle):
    """Workload 3 with the row-matching step (vector-based LZ) in front of the entropy coder: on every table, and on
    the tables Eq. 2 picks for two network bandwidths (the offline compressor selection of Section III-D, with the
    whole payload as the sample and the whole-call rates of each choice as its throughputs)."""
    T, B, D = d.shape
    nbytes = d.numel() * 4
    out = torch.zeros(nbytes, dtype=torch.uint8, device=d.device)
    sizes = torch.zeros(1 + T, dtype=torch.int64, device=d.device)
    rec = torch.empty_like(d)

    def timed(fn, reps=20):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(3):
            fn()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / reps

    def run(ctx):
        c_ms = timed(lambda: ctx.compress(d, out, sizes))
        assert ctx.sync_status() == 0
        sz = sizes.cpu().numpy().astype(np.float64)
        total = int(sz[0])
        d_ms = timed(lambda: ctx.decompress(out, total, rec))
        assert ctx.sync_status() == 0
        return {"total": total, "per_table": sz[1:], "tc": nbytes / c_ms / 1e6, "td": nbytes / d_ms / 1e6}

    ctx = b.Context(b.make_config(b.F32, T, B, D, chunk_symbols=S, flags=b.FLAG_ROW_MATCH))
    ctx.set_error_bounds(eb=ebs)
    pctx = b.Context(b.make_config(b.F32, T, B, D, chunk_symbols=S))
    pctx.set_error_bounds(eb=ebs)
    plain = run(pctx)
    lz = run(ctx)
    refs = ctx.read_row_refs()
    coded = float((refs == np.arange(B, dtype=np.uint32)[None, :]).mean())
    eb_t = torch.from_numpy(np.asarray(ebs, np.float64)).to(d.device).view(T, 1, 1)
    ok = bool(((d.double() - rec.double()).abs() <= eb_t * (1 + 1e-6)).all())
    rows = [{"workload": "3 with row matching on every table", "payload_MiB": round(nbytes / 2 ** 20, 3),
             "compression_ratio": round(nbytes / lz["total"], 3), "compress_GBps": round(lz["tc"], 2),
             "decompress_GBps": round(lz["td"], 2), "coded_rows_fraction": round(coded, 4), "bound_held": ok}]
    if with_oracle:
        import oracle
        k = 3      # one table against the oracle here (the parity tests compare whole containers)
        o = oracle.compress(d[k:k + 1].cpu().numpy(), ebs[k:k + 1], S=S, row_match=True)
        rows[0]["table_bytes_equal_oracle"] = bool(o.rc == 0 and int(o.sizes[1]) == int(lz["per_table"][k]))
    for net in (25.0, 400.0):      # GB/s per GPU: a 200 Gb/s NIC; about half of the seven xGMI links
        # the library's selection procedure (Section III-D): both compressors on the sample (here the whole payload),
        # Eq. 2 per table with the whole-call rates measured above, the choice installed in the context
        pick, _ = ctx.select_compressors(d, out, sizes, net, tc_gbps=(plain["tc"], lz["tc"]), td_gbps=(plain["td"], lz["td"]))
        pick = [int(v) for v in pick]
        hy = run(ctx)
        rows.append({"workload": f"3 hybrid: row matching where Eq. 2 prefers it at {net:g} GB/s network",
                     "payload_MiB": round(nbytes / 2 ** 20, 3), "tables_with_row_matching": int(sum(pick)),
                     "compression_ratio": round(nbytes / hy["total"], 3), "compress_GBps": round(hy["tc"], 2),
                     "decompress_GBps": round(hy["td"], 2),
                     "speedup_estimate": round(b.dlc_speedup_estimate(nbytes / hy["total"], net, hy["tc"], hy["td"]), 3),
                     "speedup_estimate_entropy_coder_only": round(b.dlc_speedup_estimate(nbytes / plain["total"], net, plain["tc"], plain["td"]), 3)})
    return rows


def all_workloads(b, torch, np, W, dev, S, with_oracle, long_form=False):
    """The five synthetic workloads, one row each (two for workload 4: fp32 and fp16; three for workload 5: the forward
    payload at the start and after the decay phase, the backward payload).  long_form: the oracle over whole payloads
    instead of a sample of tables, and the rows on destinations, row matching and a run of iterations."""
    rows = []
    sample = None if long_form else ORACLE_SAMPLE_BYTES

    def bounds(d, meta, mode, probe_frac=None, probe_abs=None, iteration=0, decay=False, rel_floor=0.0, clamp=(0.0, 0.0)):
        T = d.shape[0]
        ctx = b.Context(b.make_config(b.F16 if d.dtype == torch.float16 else b.F32, *d.shape, chunk_symbols=S))
        if probe_abs is not None:
            probe = np.full(T, probe_abs, np.float32)
        else:
            lo = d.float().amin(dim=(1, 2)).cpu().numpy()
            hi = d.float().amax(dim=(1, 2)).cpu().numpy()
            probe = (probe_frac * (hi - lo)).astype(np.float32)
        st = ctx.stats(d, probe)
        p = b.ControllerParams(mode=mode, decay_kind=b.DECAY_STEPWISE if decay else b.DECAY_NONE,
                               global_eb=meta["global_eb"], alpha=meta["alpha"], beta=meta["beta"], h_large=0.0,
                               h_small=0.05, decay_start=0, decay_len=100 if decay else 0, decay_steps=5 if decay else 0,
                               reserved=0, decay_mult0=2.0 if decay else 1.0, eb_min=clamp[0], eb_max=clamp[1],
                               rel_floor=rel_floor)
        ebs, _ = ctx.set_error_bounds(stats=st, params=p, iteration=iteration)
        return ebs

    w = W.workload1()
    d = torch.from_numpy(w.payload).to(dev)
    rows.append(_measure(b, torch, np, "1: 1 table, 256 lookups x 16, absolute bound 1e-3", d,
                         np.full(1, w.meta["eb"], np.float32), S, with_oracle, sample))
    w = W.workload2()
    d = torch.from_numpy(w.payload).to(dev)
    ebs = bounds(d, w.meta, 0, probe_abs=w.meta["global_eb"], clamp=(w.meta["eb_min"], w.meta["eb_max"]))
    rows.append(_measure(b, torch, np, "2: 26 tables x 4096 x 64, controller with absolute bounds", d, ebs, S, with_oracle, sample))
    w = W.workload3(device=dev)
    ebs = bounds(w.payload, w.meta, 1, probe_frac=0.03)
    rows.append(_measure(b, torch, np, "3: 128 x 8192 x 128, range-relative 0.03", w.payload, ebs, S, with_oracle, sample))
    if long_form:
        for n_dest in (8, 32):
            rows.append(_measure_split(b, torch, np, w.payload, ebs, S, n_dest, with_oracle))
        rows.extend(_measure_rows(b, torch, np, w.payload, ebs, S, with_oracle))
    del w
    torch.cuda.empty_cache()
    w = W.workload4(device=dev)
    ebs = bounds(w.payload, w.meta, 1, probe_frac=0.03)
    rows.append(_measure(b, torch, np, "4: 64 x 16384 x 128 multi-hot, fp32", w.payload, ebs, S, with_oracle, sample))
    h = w.meta["payload_f16"]
    ebs = bounds(h, w.meta, 1, probe_frac=0.03, rel_floor=w.meta["rel_floor_f16"])
    rows.append(_measure(b, torch, np, "4: the same sums in fp16, floor 2^-10 of the range", h, ebs, S, with_oracle, sample))
    del w, h
    torch.cuda.empty_cache()
    gen = W.Workload5(device=dev)
    fwd, bwd = gen.step()
    fwd, bwd = fwd.clone(), bwd.clone()
    for it, tag in ((0, "iteration 0 (bound x2)"), (100, "iteration 100 (bound x1)")):
        ebs = bounds(fwd, gen.meta, 1, probe_frac=0.03, iteration=it, decay=True)
        rows.append(_measure(b, torch, np, "5: forward payload, " + tag, fwd, ebs, S, with_oracle, sample))
    ebs = bounds(bwd, gen.meta, 1, probe_abs=1e-5, iteration=100, decay=True)
    rows.append(_measure(b, torch, np, "5: backward payload N(0, 1e-4)", bwd, ebs, S, with_oracle, sample))
    del gen, fwd, bwd
    torch.cuda.empty_cache()
    if long_form:
        rows.append(_run_schedule(b, torch, np, W, dev, S))
    return rows


def _run_schedule(b, torch, np, W, dev, S, iterations=200):
    """Workload 5 as a run: forward and backward payload of every iteration compressed and decompressed, bounds from
    the statistics of iteration 0 and the stepwise schedule; both compress paths over the same sequence of payloads."""
    row = {"workload": f"5: {iterations} iterations, forward + backward payload each, stepwise schedule"}
    for key, flags in (("", 0), ("carried_", b.FLAG_CARRY_CODEBOOK)):
        gen = W.Workload5(device=dev)
        T, B, D = gen.T, gen.B, gen.D
        nbytes = T * B * D * 4
        cf = b.Context(b.make_config(b.F32, T, B, D, chunk_symbols=S, flags=flags))
        cb = b.Context(b.make_config(b.F32, T, B, D, chunk_symbols=S, flags=flags))
        out = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
        sizes = torch.zeros(1 + T, dtype=torch.int64, device=dev)
        rec = torch.zeros((T, B, D), dtype=torch.float32, device=dev)
        p = b.ControllerParams(mode=1, decay_kind=b.DECAY_STEPWISE, global_eb=gen.meta["global_eb"], alpha=gen.meta["alpha"],
                               beta=gen.meta["beta"], h_large=0.0, h_small=0.05, decay_start=0, decay_len=gen.meta["decay_len"],
                               decay_steps=gen.meta["decay_steps"], reserved=0, decay_mult0=gen.meta["decay_mult0"],
                               eb_min=0.0, eb_max=0.0, rel_floor=0.0)
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(iterations)]
        comp_bytes = 0
        worst = 0.0
        for it in range(iterations):
            fwd, bwd = gen.step()
            if it == 0:
                lo, hi = fwd.amin(dim=(1, 2)).cpu().numpy(), fwd.amax(dim=(1, 2)).cpu().numpy()
                stf = cf.stats(fwd, (0.03 * (hi - lo)).astype(np.float32))
                stb = cb.stats(bwd, np.full(T, 1e-5, np.float32))
                _, cls0 = cf.set_error_bounds(stats=stf, params=p, iteration=0)
            ebf, _ = cf.set_error_bounds(stats=stf, params=p, class_override=cls0, iteration=it)
            ebb, _ = cb.set_error_bounds(stats=stb, params=p, iteration=it)
            e = ev[it]
            e[0].record()
            cf.compress(fwd, out, sizes)
            e[1].record()
            cf.decompress(out, out.numel(), rec)
            e[2].record()
            if it % 20 == 0 or it == iterations - 1:   # the bound, on the way (the parity tests check every element)
                comp_bytes_f = int(sizes[0].item())
                eb_t = torch.from_numpy(ebf.astype(np.float64)).to(dev).view(T, 1, 1)
                worst = max(worst, float(((fwd.double() - rec.double()).abs() / eb_t).max().item()))
            else:
                comp_bytes_f = None
            e[3].record()
            cb.compress(bwd, out, sizes)
            e[4].record()
            cb.decompress(out, out.numel(), rec)
            e[5].record()
            if comp_bytes_f is not None:
                comp_bytes += comp_bytes_f + int(sizes[0].item())
        torch.cuda.synchronize()
        assert cf.sync_status() == 0 and cb.sync_status() == 0
        c_ms = sum(e[0].elapsed_time(e[1]) + e[3].elapsed_time(e[4]) for e in ev)
        d_ms = sum(e[1].elapsed_time(e[2]) + e[4].elapsed_time(e[5]) for e in ev)
        n_sampled = len([it for it in range(iterations) if it % 20 == 0 or it == iterations - 1])
        moved = 2.0 * nbytes * iterations
        row[key + "compress_GBps"] = round(moved / c_ms / 1e6, 2)
        row[key + "decompress_GBps"] = round(moved / d_ms / 1e6, 2)
        row[key + "compression_ratio_sampled"] = round(2.0 * nbytes * n_sampled / comp_bytes, 3)
        row[key + "worst_error_over_bound"] = round(worst, 6)
        del gen, cf, cb
        torch.cuda.empty_cache()
    row["payload_MiB"] = round(2.0 * nbytes * iterations / 2 ** 20, 1)
    return row


if __name__ == "__main__":
    main()
