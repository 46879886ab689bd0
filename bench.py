#!/usr/bin/env python3
"""Benchmark of the SVGD all-particle update on one MI355X.

A "step" is one svgd_step call: Gram / pairwise-d2 pass, partial reduction, median bandwidth + K,
fused in-place update - the whole hot path - over one synthetic particle population already
resident in HBM.  Prints ONE JSON line (see README/DESIGN for the fields).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published

# HBM traffic of the dominant kernel from rocprofv3 --pmc (see profiles/): average KiB per launch
# as FETCH_SIZE / WRITE_SIZE report it, and the factors that the same counters need to reproduce
# the known size of the plain copy kernel (svgd_diag_copy).  The numbers belong to one version of
# the kernel source: if the hash below no longer matches, "traffic" is reported as null.
TRAFFIC_COUNTERS = {
    # (config, carried Gram?, rows padded to 32 floats?) -> (FETCH_SIZE KiB, WRITE_SIZE KiB)
    (5, True, True): (2801879.6, 2795580.1),
    (5, False, True): (2801515.4, 2793492.0),
    (5, True, False): (4072296.5, 2797113.5),   # mean of the two walking directions (separate instances)
    (5, False, False): (4066961.6, 2795026.6),
    (3, True, True): (253521.8, 250530.1),      # D = 2,000,000 is a multiple of 32: ld = D either way
    (3, False, True): (253579.1, 250000.0),
    (3, True, False): (253532.1, 250530.1),
    (3, False, False): (253573.5, 250000.0),
    (4, True, True): (353133.5, 350745.0),
    (4, False, True): (359983.7, 352893.9),
    (4, True, False): (366806.0, 356675.6),
    (4, False, False): (365467.2, 354787.4),
}
TRAFFIC_SCALE = (2.0, 1.0)     # FETCH_SIZE counts half of the bytes a plain copy reads, WRITE_SIZE all
TRAFFIC_SOURCE_SHA256 = "4a8b61cedc15aec6e84aa11f16da428b8a6b241d90624b332ae90d20edc9ee1c"


def kernel_source_hash():
    import hashlib
    d = os.path.join(ROOT, "paper_2306_06528_amd", "csrc")
    h = hashlib.sha256()
    for name in ("update_kernels.hpp", "bandwidth_kernels.hpp", "common.hpp"):
        with open(os.path.join(d, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


UPDATE_BYTES_PER_PARAM = 12    # read X, read G, write X
STEP_BYTES_PER_PARAM = 16      # + the Gram pass reads X once more


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(wl):
    """Times the fp64 CPU oracle as it stands on a bounded column sample of the same workload."""
    import numpy as np
    from oracle import svgd_oracle
    n = wl.n
    # the oracle costs O(n^2) per column: 12M columns at n=64 are about 100 core-seconds
    ds = int(min(wl.D, max(4096, 12_000_000 * 64 // max(n, 4))))
    Xs = wl.X0[:, :ds].contiguous().cpu().numpy()
    Gs = wl.score(wl.X0, 0)[:, :ds].contiguous().cpu().numpy()
    reps, dt = 0, 0.0
    t0 = time.perf_counter()
    while reps < 1 or (dt < 10.0 and reps < 1000):   # at least one step, then about 10 s of them
        svgd_oracle.step(Xs, Gs, wl.cfg.eps, want_phi=False, want_xnew=True)
        reps += 1
        dt = time.perf_counter() - t0
    return {
        "value": n * ds * reps / dt,
        "unit": "particle-params/s",
        "cores": svgd_oracle.num_threads(),
        "cpu": cpu_model(),
        "kind": "oracle",
        "sample": f"{reps} fp64 oracle step(s) on the first {ds} of {wl.D} columns, all {n} particles "
                  f"({dt:.1f} s)",
    }


def run_swag(args, wl, X, svgd, torch):
    """One "step" = one swag_update_moments call over all n x D parameters (20 B per parameter)."""
    n, D = wl.n, wl.D
    mean = torch.zeros_like(X)
    sq = torch.zeros_like(X)
    for t in range(args.warmup):
        svgd.swag_update_moments(mean, sq, X, t)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for t in range(args.steps):
        svgd.swag_update_moments(mean, sq, X, args.warmup + t)
    e1.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kern_ms = e0.elapsed_time(e1) / args.steps     # back-to-back launches of the one kernel
    gbs = 20 * n * D / (kern_ms * 1e-3) / 1e9
    out = {
        "metric": "multi-SWAG particle-params absorbed into running moments/s",
        "value": n * D * args.steps / dt, "unit": "particle-params/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{wl.cfg.name}: moments of n={n} particles x D={D} fp32", "n": n, "D": D,
                   "config_index": args.config},
        "roofline": {"kernel": "swag_moments_kernel", "bound": "hbm", "achieved": gbs,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS, "traffic": None},
    }
    if not args.no_cpu_baseline:
        import numpy as np
        from oracle import svgd_oracle
        ds = int(min(D, 4_000_000))
        Xs = X[:, :ds].contiguous().cpu().numpy()
        m = np.zeros(Xs.shape)
        s2 = np.zeros(Xs.shape)
        c0 = time.perf_counter()
        reps = 4
        for t in range(reps):
            svgd_oracle.swag_update(m, s2, Xs, t)
        cdt = time.perf_counter() - c0
        out["cpu_baseline"] = {"value": n * ds * reps / cdt, "unit": "particle-params/s",
                               "cores": svgd_oracle.num_threads(), "kind": "oracle",
                               "sample": f"{reps} fp64 oracle updates on the first {ds} of {D} columns, "
                                         f"all {n} particles ({cdt:.1f} s)"}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20,
                    help="untimed steps first (the chip needs some 30 ms of work to reach its steady clocks)")
    ap.add_argument("--config", type=int, default=5, help="workload 1..5 (default 5: n=64, D=11,173,962)")
    ap.add_argument("--particles", type=int, default=None,
                    help="another particle count n with the config's distributions (a side measurement, "
                         "e.g. n = 33; the line then names the size it ran)")
    ap.add_argument("--params", type=int, default=None, help="another flattened size D, likewise")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--separate-gram", action="store_true",
                    help="run the pairwise-d2 pass as its own kernel every step instead of carrying "
                         "the sums over from the previous update (SVGD_FLAG_CARRY_GRAM)")
    ap.add_argument("--fuse", action="store_true",
                    help="SVGD_FLAG_FUSE_MFMA: the single-launch fused step also for 13 <= n <= 32 "
                         "(measured slower than two launches there; for the record)")
    ap.add_argument("--dense-rows", action="store_true",
                    help="rows D floats apart (ld = D) instead of ld = D rounded up to 32 floats")
    ap.add_argument("--swag", action="store_true",
                    help="time the multi-SWAG running-moments kernel on the config's n x D instead of svgd_step")
    ap.add_argument("--verbose", action="store_true", help="print the yardstick sweep to stderr")
    ap.add_argument("--no-ceiling", action="store_true",
                    help="skip the yardstick sweep (roofline.ceiling = null): keeps counter runs of a profiler short")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch the plain copy kernel once over G (for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on exactly one GPU (no sharding, no collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2306_06528_amd import svgd, workloads   # raises if libsvgd.so is missing

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    wl = workloads.make(args.config, device="cuda:0", n=args.particles, D=args.params)
    n, D, eps = wl.n, wl.D, wl.cfg.eps
    stream = torch.cuda.current_stream()

    def laid_out(t, padded):
        """(buffer, n x D view): rows ld = D rounded up to 32 floats apart (each row starts on a
        128-byte boundary), or densely packed."""
        if not padded:
            buf = t.clone()
            return buf, buf
        buf = svgd.padded_rows(n, D, device=t.device)
        buf.copy_(t)
        return buf, buf

    padded = not args.dense_rows
    G0 = wl.score(wl.X0, 0)
    _, X = laid_out(wl.X0, padded)
    _, G = laid_out(G0, padded)
    ld = X.stride(0) if n > 1 else D

    if args.swag:
        run_swag(args, wl, wl.X0.clone(), svgd, torch)
        return

    if args.calibrate_copy:
        scratch = torch.empty_like(G0)
        svgd.diag_copy(scratch, G0, stream=stream)
        torch.cuda.synchronize()
        del scratch

    def timed(flags, Xv, Gv, kinds=None, per_step=False):
        """Warm-up, then K timed steps.  `kinds`: kernels of these kinds are bracketed by HIP
        events on the launch stream during the timed steps (recorded by the library from a pool
        created beforehand; two event records per timed kernel, a few microseconds each).
        per_step: one event per step boundary on the launch stream instead (step-to-step times).
        Returns (wall seconds, {kind: (ms, launches)} or None, per-launch or per-step ms list)."""
        with svgd.Svgd(n, D, 0, flags=flags) as eng:
            for _ in range(args.warmup):
                eng.step(Xv, Gv, eps, stream=stream)
            marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)] if per_step else None
            if kinds:
                eng.profile_begin(kinds)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for k in range(args.steps):
                if per_step:
                    marks[k].record(stream)
                eng.step(Xv, Gv, eps, stream=stream)
            if per_step:
                marks[-1].record(stream)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            prof, recs = eng.profile_end_records() if kinds else (None, None)
            if per_step:
                recs = [marks[k].elapsed_time(marks[k + 1]) for k in range(args.steps)]
        return dt, prof, recs

    def stats(ms_list):
        v = sorted(ms_list)
        return {"median": v[len(v) // 2] if len(v) % 2 else 0.5 * (v[len(v) // 2 - 1] + v[len(v) // 2]),
                "min": v[0], "max": v[-1], "mean": sum(v) / len(v)}

    def triad_ceiling(Xv, Gv):
        """What the memory system gives the update's traffic and nothing else: x += s*g in place
        over the same row streams of the same buffers (s = 0: X keeps its values), best of the
        access patterns (two shapes, two depths, with and without streaming loads) and grid sizes.  GB/s at 12 bytes per element."""
        cus = torch.cuda.get_device_properties(0).multi_processor_count
        best = None
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 10
        # every variant both ways: always from the near end, and (pattern + 16 on every other call)
        # alternating the direction as the steps of a CARRY_GRAM handle do
        for pattern in [p + 16 * alt for p in range(12) for alt in (0, 1)]:
            for per_cu in (1, 2, 4, 8):
                for i in range(4):
                    svgd.diag_axpy_rows(Xv, Gv, 0.0, pattern ^ (16 * (i & 1) if pattern >= 16 else 0), cus * per_cu, stream=stream)
                e0.record(stream)
                for i in range(reps):
                    svgd.diag_axpy_rows(Xv, Gv, 0.0, pattern ^ (16 * (i & 1) if pattern >= 16 else 0), cus * per_cu, stream=stream)
                e1.record(stream)
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / reps
                gbs = UPDATE_BYTES_PER_PARAM * n * D / (ms * 1e-3) / 1e9
                if args.verbose:
                    print(f"axpy_rows pattern {pattern} x {per_cu}/CU: {ms:.4f} ms {gbs:.0f} GB/s", file=sys.stderr)
                if best is None or gbs > best["gbs"]:
                    best = {"gbs": gbs, "ms": ms, "pattern": pattern, "workgroups": cus * per_cu}
        return best

    def read_ceiling(Xv):
        """What the memory system gives the pairwise pass's traffic and nothing else: every element
        of X read once (svgd_diag_read_rows), best of the two access shapes, with and without
        streaming loads, and of four grid sizes.  GB/s at 4 bytes per element."""
        cus = torch.cuda.get_device_properties(0).multi_processor_count
        best = None
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 10
        for pattern in range(4):
            for per_cu in (1, 2, 4, 8):
                sink = torch.empty(cus * per_cu, device=Xv.device)
                for _ in range(3):
                    svgd.diag_read_rows(Xv, sink, pattern, stream=stream)
                e0.record(stream)
                for _ in range(reps):
                    svgd.diag_read_rows(Xv, sink, pattern, stream=stream)
                e1.record(stream)
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / reps
                gbs = 4 * n * D / (ms * 1e-3) / 1e9
                if args.verbose:
                    print(f"read_rows pattern {pattern} x {per_cu}/CU: {ms:.4f} ms {gbs:.0f} GB/s", file=sys.stderr)
                if best is None or gbs > best["gbs"]:
                    best = {"gbs": gbs, "ms": ms, "pattern": pattern, "workgroups": cus * per_cu}
        return best

    carry = not args.separate_gram
    flags = svgd.FLAG_CARRY_GRAM if carry else 0
    if args.fuse:
        flags |= svgd.FLAG_FUSE_MFMA
    # the timed region: K steps, the dominant kernel (update) timed by events inside it
    dt, prof_upd, recs_upd = timed(flags, X, G, kinds=("update",))
    # the same K steps again: with every kernel timed (the per-kernel breakdown), with one event
    # per step (median / min step time), and with no events at all (what the events cost)
    _, prof, _ = timed(flags, X, G, kinds=svgd.KERNEL_KINDS)
    _, _, step_ms = timed(flags, X, G, per_step=True)
    dt_plain, _, _ = timed(flags, X, G)
    ceiling = None if args.no_ceiling else triad_ceiling(X, G)

    def side(res, bytes_per_param, **what):
        dt_side = res[0]
        what.update({"ms_per_step": dt_side * 1e3 / args.steps, "value": n * D * args.steps / dt_side,
                     "step_hbm_frac": bytes_per_param * n * D / (dt_side / args.steps) / 1e9 / HBM_PEAK_GBS})
        return what

    # for reference, the same workload (a) with the pairwise-d2 pass as its own kernel every step,
    # (b) with densely packed rows (ld = D), (c) both: the plain svgd_step(X, G, n, D, eps, stream)
    # of the four-call ABI on a handle without flags - 16 bytes per particle-param
    alt = None
    gram_ms_sep = None
    if carry:
        alt = side(timed(0, X, G), STEP_BYTES_PER_PARAM, gram="separate pass")
        res = timed(0, X, G, kinds=("gram",))
        if res[1]["gram"][1] > 0:
            gram_ms_sep = res[1]["gram"][0] / res[1]["gram"][1]
    alt_dense = alt_plain = None
    if padded:
        _, Xd = laid_out(wl.X0, False)
        _, Gd = laid_out(G0, False)
        if ld != D:
            alt_dense = side(timed(flags, Xd, Gd), UPDATE_BYTES_PER_PARAM if carry else STEP_BYTES_PER_PARAM, ld=D)
        alt_plain = side(timed(0, Xd, Gd), STEP_BYTES_PER_PARAM, ld=D, gram="separate pass",
                         call="svgd_step(handle, X, G, n, D, eps, stream), handle flags = 0")
        res = timed(0, Xd, Gd, kinds=("update",))
        u_ms = res[1]["update"][0] / max(res[1]["update"][1], 1)
        alt_plain["update_kernel_ms"] = u_ms
        alt_plain["update_kernel_hbm_frac"] = UPDATE_BYTES_PER_PARAM * n * D / (u_ms * 1e-3) / 1e9 / HBM_PEAK_GBS
        del Xd, Gd

    assert torch.isfinite(X).all().item(), "X went non-finite during the benchmark"
    ms_per_step = dt * 1e3 / args.steps
    value = n * D * args.steps / dt
    kern_ms = {k: (ms / max(c, 1)) for k, (ms, c) in prof.items()}
    upd_ms = prof_upd["update"][0] / max(prof_upd["update"][1], 1)   # over the timed steps
    upd_gbs = UPDATE_BYTES_PER_PARAM * n * D / (upd_ms * 1e-3) / 1e9
    gram_gbs = 4 * n * D / (kern_ms["gram"] * 1e-3) / 1e9 if kern_ms["gram"] > 0 else None
    # the pairwise pass as its own kernel (this run's, or the separate-pass alternative's) against
    # the peak and against a plain read of the same rows
    gram_ms = kern_ms["gram"] if kern_ms["gram"] > 0 else gram_ms_sep
    gram_pass = None
    if gram_ms:
        rc = None if args.no_ceiling else read_ceiling(X)
        g_gbs = 4 * n * D / (gram_ms * 1e-3) / 1e9
        gram_pass = {"kernel_ms": gram_ms, "gbs": g_gbs, "frac": g_gbs / HBM_PEAK_GBS,
                     "read_ceiling": rc and rc["gbs"],
                     "read_ceiling_kernel": rc and (f"svgd_diag_read_rows pattern {rc['pattern']}, "
                                                    f"{rc['workgroups']} workgroups, {rc['ms']:.4f} ms"),
                     "frac_of_read_ceiling": rc and g_gbs / rc["gbs"]}

    tiny = n <= 8 and n * D <= 16384   # sizes the library runs as a single kernel
    traffic = None
    key = (args.config, carry, padded)
    resized = args.particles is not None or args.params is not None
    if not resized and key in TRAFFIC_COUNTERS and kernel_source_hash() == TRAFFIC_SOURCE_SHA256:
        f_kib, w_kib = TRAFFIC_COUNTERS[key]
        traffic = (f_kib * TRAFFIC_SCALE[0] + w_kib * TRAFFIC_SCALE[1]) * 1024.0

    out = {
        "metric": "SVGD particle-params updated/s",
        "value": value,
        "unit": "particle-params/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{wl.cfg.name}{' (resized)' if resized else ''}: n={n} particles x D={D} fp32, "
                               f"rows {ld} floats apart, eps={eps}",
                   "n": n, "D": D, "ld": ld, "config_index": args.config,
                   "gram": "carried from the previous update" if carry else "separate pass",
                   "fuse_mfma": bool(args.fuse)},
        "step_hbm_frac": (UPDATE_BYTES_PER_PARAM if carry else STEP_BYTES_PER_PARAM) * n * D
                         / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "kernel_ms": kern_ms,
        "ms_per_step_without_events": dt_plain * 1e3 / args.steps,
        "step_ms": stats(step_ms),
        "update_kernel_ms": stats([ms for _, ms in recs_upd]),
        "separate_gram": alt,
        "dense_rows": alt_dense,
        "plain_svgd_step": alt_plain,
        "gram_gbs": gram_gbs,
        "gram_pass": gram_pass,
        "roofline": {
            "kernel": "step_tiny_kernel (the whole step in one workgroup)" if tiny else
                      ("update_valu_kernel" if n <= 12 else "update_mfma_kernel") +
                      " (fused K.[G|X] in-place update" +
                      (", also accumulating the next step's pair sums)" if carry else ")"),
            "bound": "hbm",
            "achieved": upd_gbs,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": upd_gbs / HBM_PEAK_GBS,
            "traffic": traffic,
            # the same bytes moved by a kernel that does nothing else (svgd_diag_axpy_rows on the
            # same X and G, in the same run): the practical ceiling, and the update against it
            "ceiling": ceiling and ceiling["gbs"],
            "ceiling_kernel": ceiling and (f"svgd_diag_axpy_rows pattern {ceiling['pattern'] & 15}"
                                           f"{', direction alternating from call to call' if ceiling['pattern'] >= 16 else ''}, "
                                           f"{ceiling['workgroups']} workgroups, {ceiling['ms']:.4f} ms"),
            "frac_of_ceiling": ceiling and upd_gbs / ceiling["gbs"],
        },
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
