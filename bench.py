"""Benchmark of the dq8 hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Workload: the simulated data-parallel aggregation on the 61 100 840-element AlexNet-shaped
gradient bucket with block 4096 and the dynamic tree type (K = 8 workers).  One step is one
pass of the whole path over one set of buffers:

    dq8_absmax(x)  ->  dq8_encode(x)  ->  dq8_decode(codes)  ->
    dq8_decode_accumulate_avg(8 x codes)  ->  dq8_encode(mean)

Inputs are resident in HBM before the timed region.  Four distinct buffer sets (> 4 GB in
all) are used in rotation, and no call reads what the call before it wrote, so the 256 MB
last-level cache cannot serve a step from an earlier one.

value = fp32 bytes the five calls consume or produce (4 bytes x n each) per second over the
whole timed region.  The roofline object is for the kernel that takes the largest share of a
step (the K-way decode-and-average); `kernels` lists all of them, each timed with HIP events
on the launch stream around K consecutive launches of that call over the same rotating buffers.
`kernels` also times two calls that are not part of a step: dq8_decode_avg_encode (the average and
the re-compression in one call) and dq8_decode_accumulate_avg_local (a local fp32 term in the average).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
KIND = 0          # dynamic tree
BLOCK = 4096
K_WORKERS = 8
N_SETS = 4

# HBM bytes per launch of the dominant kernel measured with rocprofv3 --pmc (FETCH_SIZE and
# WRITE_SIZE runs on this script, each scaled by what the same counter reads for the calibration
# copy kernel: 1.99982 and 1.00000); the runs are recorded in profiles/hbm_traffic_bench_c5.md.
GROUPS = 5  # per-kernel timing: median of this many groups of `steps` launches
MEASURED_TRAFFIC_BYTES = {"decode_accumulate_avg": int((481267 + 238675) * 1024)}


def algorithmic_bytes(n, nb):
    """Bytes each call must move (fp32 = 4 B, code = 1 B, one fp32 scale per block)."""
    return {
        "absmax": 4 * n + 4 * nb,
        "encode": 4 * n + n + 4 * nb,
        "decode": n + 4 * nb + 4 * n,
        "decode_accumulate_avg": K_WORKERS * (n + 4 * nb) + 4 * n,
        "re_encode": 4 * n + n + 4 * nb,
        # not part of a step: the second exchange round as one call, and the average with a local fp32 term
        "decode_avg_encode": K_WORKERS * (n + 4 * nb) + n + 4 * nb,
        "decode_accumulate_avg_local": K_WORKERS * (n + 4 * nb) + 4 * n + 4 * n,
        # the approximation-error statistics with the scales handed in: one pass over the fp32 input
        "error_stats": 4 * n + 4 * nb + 32 * nb,
        # one GPU's share of the second round on an 8-GPU node: 7 received buffers + its own fp32 slice, compressed
        "decode_avg_encode_7_local": 7 * (n + 4 * nb) + 4 * n + n + 4 * nb,
        # compression into the 8-bit mantissa type (ranks of distinct magnitudes mapped to codes)
        "encode_mantissa": 4 * n + n + 4 * nb,
    }


def device_info():
    """Name, compute units and clocks of the GPU as the runtime reports them."""
    import torch
    p = torch.cuda.get_device_properties(0)
    info = {"name": p.name, "compute_units": p.multi_processor_count, "memory_GiB": round(p.total_memory / 2 ** 30, 1)}
    for key in ("clock_rate", "memory_clock_rate"):
        if hasattr(p, key):
            info[key + "_MHz"] = round(getattr(p, key) / 1000.0, 1)
    return info


def cpu_baseline(host_buckets):
    """The oracle, as it stands, timed on the host cores on one step of the same workload.

    The oracle's brute-force encoder runs at some 10^8 elements/s on 16 cores, so the bounded
    sample is one whole step on the full bucket (a few seconds) after an untimed set-up that
    oracle-encodes the eight workers' buckets.
    """
    import oracle
    cores = len(os.sched_getaffinity(0))
    threads = oracle.set_threads(cores)
    n = host_buckets[0].size
    enc = [oracle.encode(KIND, x, BLOCK) for x in host_buckets]  # the workers' buffers: set-up, not timed
    t0 = time.perf_counter()
    oracle.absmax(host_buckets[0], BLOCK)
    codes, scales = oracle.encode(KIND, host_buckets[0], BLOCK)
    oracle.decode(KIND, codes, scales, BLOCK)
    mean = oracle.decode_accumulate_avg(KIND, [e[0] for e in enc], [e[1] for e in enc], BLOCK)
    oracle.encode(KIND, mean, BLOCK)
    dt = time.perf_counter() - t0
    return {"value": round(5 * 4 * n / dt / 1e9, 4), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": "one whole step (absmax, encode, decode, 8-way decode-and-average, re-encode) on the full "
                      "%d-element bucket, %.1f s" % (n, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", default=None, help="time only this call in the event pass (profiling aid)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_1511_04561_amd import dq8, workloads

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    dq8.init()
    n = workloads.C3_NUMEL
    nb = dq8.n_blocks(n, BLOCK)

    # ---- resident inputs: 8 workers' buckets, encoded once (set-up)
    t0 = time.time()
    xw, cw, sw, host_buckets = [], [], [], []
    for w in range(K_WORKERS):
        host_buckets.append(workloads.bucket(5, worker=w))
        x = torch.from_numpy(host_buckets[-1]).cuda()
        c, s = dq8.encode(KIND, x, BLOCK)
        xw.append(x)
        cw.append(c)
        sw.append(s)
    torch.cuda.synchronize()
    print("set-up: generated and encoded %d workers in %.1f s" % (K_WORKERS, time.time() - t0), file=sys.stderr, flush=True)

    sets = []
    for r in range(N_SETS):
        st = {
            "x": xw[r],                                                    # fp32 gradients of worker r
            "codes": [c.clone() for c in cw], "scales": [s.clone() for s in sw],   # the 8 received buffers
            "amax": torch.empty(nb, dtype=torch.float32, device="cuda"),
            "c_out": torch.empty(n, dtype=torch.uint8, device="cuda"),
            "s_out": torch.empty(nb, dtype=torch.float32, device="cuda"),
            "dec": torch.empty(n, dtype=torch.float32, device="cuda"),
            "mean": torch.empty(n, dtype=torch.float32, device="cuda"),
            "rc": torch.empty(n, dtype=torch.uint8, device="cuda"),
            "rs": torch.empty(nb, dtype=torch.float32, device="cuda"),
            "stats": torch.empty((nb, 4), dtype=torch.float64, device="cuda"),
            "means": torch.empty(2, dtype=torch.float64, device="cuda"),
        }
        sets.append(st)
    for st in sets:  # every mean buffer holds a valid average before it is re-encoded
        dq8.decode_accumulate_avg(KIND, st["codes"], st["scales"], BLOCK, out=st["mean"])
    torch.cuda.synchronize()

    def calls(i):
        st, nxt = sets[i % N_SETS], sets[(i + 1) % N_SETS]
        return [
            ("absmax", lambda: dq8.absmax(st["x"], BLOCK, scales=st["amax"])),
            ("encode", lambda: dq8.encode(KIND, st["x"], BLOCK, scales=st["s_out"], codes=st["c_out"])),
            ("decode", lambda: dq8.decode(KIND, st["codes"][0], st["scales"][0], BLOCK, out=st["dec"])),
            ("decode_accumulate_avg", lambda: dq8.decode_accumulate_avg(KIND, st["codes"], st["scales"], BLOCK, out=st["mean"])),
            # the mean written one step earlier in the rotation (long evicted), not the one just produced
            ("re_encode", lambda: dq8.encode(KIND, nxt["mean"], BLOCK, scales=st["rs"], codes=st["rc"])),
        ]

    def extra_calls(i):
        """Calls beside the step: timed per kernel only."""
        st, nxt = sets[i % N_SETS], sets[(i + 1) % N_SETS]
        return [
            ("decode_avg_encode", lambda: dq8.decode_avg_encode(KIND, st["codes"], st["scales"], BLOCK,
                                                                scales=st["rs"], codes=st["rc"])),
            ("decode_accumulate_avg_local", lambda: dq8.decode_accumulate_avg(KIND, st["codes"], st["scales"], BLOCK,
                                                                              out=st["dec"], local=nxt["x"])),
            ("error_stats", lambda: dq8.error_stats(KIND, st["x"], BLOCK, scales=st["s_out"], scales_given=True,
                                                    stats=st["stats"], means=st["means"])),
            ("decode_avg_encode_7_local", lambda: dq8.decode_avg_encode(KIND, st["codes"][:7], st["scales"][:7], BLOCK,
                                                                        local=nxt["x"], scales=st["rs"], codes=st["rc"])),
            ("encode_mantissa", lambda: dq8.encode(dq8.MANTISSA, st["x"], BLOCK, scales=st["rs"], codes=st["rc"])),
        ]

    def step(i):
        for _, f in calls(i):
            f()

    # ---- timed region: W warm-up steps, then exactly K steps between synchronisations
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    fp32_bytes_per_step = 5 * 4 * n
    value = fp32_bytes_per_step / (elapsed / args.steps) / 1e9

    # ---- per-kernel durations: the same calls again, one kernel at a time: HIP events on the launch
    # stream bracket `steps` consecutive launches of that call, rotating through the buffer sets exactly
    # as the steps above do, so launch gaps are amortised and the cache still cannot help.
    def all_calls(i):
        return calls(i) + extra_calls(i)

    names = [nm for nm, _ in all_calls(0)]
    if args.only:
        names = [nm for nm in names if nm == args.only]
    tot = {}
    for idx, nm in enumerate([nm for nm, _ in all_calls(0)]):
        if nm not in names:
            continue
        for i in range(3):
            all_calls(i)[idx][1]()
        groups = []
        for g in range(GROUPS):  # median over several groups of `steps` consecutive launches
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for i in range(args.steps):
                all_calls(3 + g * args.steps + i)[idx][1]()
            b.record()
            torch.cuda.synchronize()
            groups.append(a.elapsed_time(b))
        tot[nm] = sorted(groups)[len(groups) // 2]
    alg = algorithmic_bytes(n, nb)
    kernels = {}
    for nm in names:
        ms = tot[nm] / args.steps
        gbps = alg[nm] / (ms * 1e-3) / 1e9
        kernels[nm] = {"ms": round(ms, 5), "fp32_GBps": round(4 * n / (ms * 1e-3) / 1e9, 1),
                       "hbm_GBps": round(gbps, 1), "frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4),
                       "algorithmic_bytes": alg[nm]}

    # ---- calibration: plain copy with the same access pattern (context for the fractions above)
    ca, cb_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(4):
        dq8.calibration_copy(sets[i % N_SETS]["dec"], sets[(i + 1) % N_SETS]["x"])
    ca.record()
    reps = 20
    for i in range(reps):
        dq8.calibration_copy(sets[i % N_SETS]["dec"], sets[(i + 1) % N_SETS]["x"])
    cb_.record()
    torch.cuda.synchronize()
    copy_gbps = 8 * n / (ca.elapsed_time(cb_) / reps * 1e-3) / 1e9

    dom = "decode_accumulate_avg" if "decode_accumulate_avg" in kernels else names[0]
    roof = {"bound": "hbm", "kernel": dom, "achieved": kernels[dom]["hbm_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": kernels[dom]["frac_of_peak"], "traffic": MEASURED_TRAFFIC_BYTES.get(dom),
            "algorithmic_bytes_per_launch": alg[dom], "avg_launch_ms": kernels[dom]["ms"]}

    out = {
        "metric": "GB/s of fp32 gradients encoded/decoded (and % of HBM peak) on 1 MI355X",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "C5: K=8 workers x 61100840-element AlexNet-shaped gradient bucket, block=4096, "
                               "dynamic tree; step = absmax + encode + decode + decode_accumulate_avg(K=8) + re-encode",
                   "n": n, "block": BLOCK, "K": K_WORKERS, "kind": "dynamic_tree", "buffer_sets": N_SETS},
        "roofline": roof,
        "kernels": kernels,
        "kernel_timing": "median of %d groups of %d consecutive launches between HIP events" % (GROUPS, args.steps),
        "device": device_info(),
        "copy_kernel_GBps": round(copy_gbps, 1),
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(host_buckets)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
