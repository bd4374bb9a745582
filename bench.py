"""Benchmark of the dq8 hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--only CALL] [--no-cpu-baseline]
    python bench.py --sweep [blocks,workers,configs]

Workload of the default run: the simulated data-parallel aggregation on the 61 100 840-element
AlexNet-shaped gradient bucket with block 4096 and the dynamic tree type (K = 8 workers).  One step is
one pass of the whole path:

    dq8_absmax(x)  ->  dq8_encode(x')  ->  dq8_decode(codes)  ->
    dq8_decode_accumulate_avg(8 x codes')  ->  dq8_encode(mean'')

Inputs are resident in HBM before the timed region.  Four distinct buffer sets (> 4 GB in all) are used
in rotation, and within a step every call reads from a different set than its neighbours (x of set i for
the maximum, x of set i + 1 for the compression, codes of set i for the decompression, codes of set i + 1
for the average, the mean that was written two steps earlier for the re-compression): no call reads
anything that either of the two calls before it read or wrote, and whatever a call reads was last touched
more than 1 GB of traffic ago, so the 256 MB last-level cache cannot serve any of it.

Order of a run: untimed clock-settling steps (groups of ten until three consecutive groups agree within
1 %; their number is reported), W untimed warm-up steps, exactly K timed steps between two
synchronisations.  value = fp32 bytes the five calls consume or produce (4 bytes x n each) per second over
the timed region.

`kernels` times every call on its own: 200 untimed launches of that call (the clocks follow a change of load with a
delay), then HIP events on the launch stream around max(K, 50) consecutive launches of it over the same rotating
buffers, median of five such groups.  It also holds calls that
are not part of a step (the one-call second round, the local fp32 term, the error statistics, the mantissa
type).  `roofline` is for the call that takes the largest share of a step (the K-way decode-and-average);
its `traffic` is the HBM traffic per launch recorded in profiles/hbm_traffic_bench_c5.md (rocprofv3
counters of an earlier run of this script, not measured in this run).

--sweep prints one JSON line per measurement instead (not part of `value`): every call at other block
lengths and worker counts on the same bucket, and the small configurations C1 (MLP gradients, one scale
per tensor), C2 (convnet gradients, one scale per tensor, three data types) and C4 (activations, one scale
per row) as per-tensor calls over enough copies of the configuration to exceed 1 GB, each pass also recorded into
a HIP graph and replayed, and C1 / C2 also as one array with one call for all tensors (dq8_encode_segments,
dq8_decode_segments).
"""
import argparse
import itertools
import json
import os
import re
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
GROUPS = 5        # per-kernel timing: median of this many groups of consecutive launches
# untimed launches of a call before its timed groups: the clocks follow the load with a delay of tens of milliseconds, and a
# call that keeps the vector units busy reads up to 10 % slow when it is timed right after calls that only move data
PRIME = 200
MIN_LAUNCHES = 50  # launches per group, at least

TRAFFIC_PROFILE = os.path.join("profiles", "hbm_traffic_bench_c5.md")
# the row of that file for the kernel behind each call (kernel name as the profiler prints it)
TRAFFIC_ROW = {"decode_accumulate_avg": r"k_decode_avg_full<8, [^|]*false>"}


def recorded_traffic(call):
    """HBM bytes per launch of the kernel behind `call` as recorded in TRAFFIC_PROFILE (scaled read +
    scaled write KiB columns), or None when the file has no such row."""
    pattern = TRAFFIC_ROW.get(call)
    path = os.path.join(ROOT, TRAFFIC_PROFILE)
    if not pattern or not os.path.exists(path):
        return None
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 5 and re.fullmatch(pattern, cells[0]):
            return int((float(cells[3]) + float(cells[4])) * 1024)
    return None


def algorithmic_bytes(n, nb, K=K_WORKERS):
    """Bytes each call must move (fp32 = 4 B, code = 1 B, one fp32 scale per block)."""
    return {
        "absmax": 4 * n + 4 * nb,
        "encode": 4 * n + n + 4 * nb,
        "decode": n + 4 * nb + 4 * n,
        "decode_accumulate_avg": K * (n + 4 * nb) + 4 * n,
        "re_encode": 4 * n + n + 4 * nb,
        # not part of a step: the second exchange round as one call, and the average with a local fp32 term
        "decode_avg_encode": K * (n + 4 * nb) + n + 4 * nb,
        "decode_accumulate_avg_local": K * (n + 4 * nb) + 4 * n + 4 * n,
        # the approximation-error statistics with the scales handed in: one pass over the fp32 input
        "error_stats": 4 * n + 4 * nb + 32 * nb,
        # one GPU's share of the second round on an 8-GPU node: 7 received buffers + its own fp32 slice, compressed
        "decode_avg_encode_7_local": 7 * (n + 4 * nb) + 4 * n + n + 4 * nb,
        # compression into the 8-bit mantissa type
        "encode_mantissa": 4 * n + n + 4 * nb,
    }


def device_info(internal):
    """Name, memory, compute units and peak clocks of the GPU as the runtime reports them."""
    import torch
    p = torch.cuda.get_device_properties(0)
    info = {"name": p.name, "memory_GiB": round(p.total_memory / 2 ** 30, 1)}
    info.update(internal.device_info())
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


def event_time_ms(torch, launch, launches, groups=GROUPS, prime=3):
    """Median over `groups` of the time of `launches` consecutive launch(i) calls between two HIP events on the
    current stream, per launch, in milliseconds.  i keeps counting so that buffer rotation continues."""
    for i in range(prime):
        launch(i)
    times = []
    for g in range(groups):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(launches):
            launch(prime + g * launches + i)
        b.record()
        torch.cuda.synchronize()
        times.append(a.elapsed_time(b) / launches)
    return sorted(times)[len(times) // 2]


def copy_rate_gbps(torch, internal, srcs, dsts, n):
    """The plain copy kernel with the codec kernels' access pattern over rotating buffers: GB/s of 8 bytes per element."""
    ms = event_time_ms(torch, lambda i: internal.calibration_copy(dsts[i % len(dsts)], srcs[(i + 1) % len(srcs)]), 20, groups=3)
    return 8 * n / (ms * 1e-3) / 1e9


class Bucket:
    """The C5 buffers: K workers' fp32 buckets, and N_SETS sets of received codes / scales and outputs."""

    def __init__(self, torch, dq8, workloads, keep_host=True):
        self.torch, self.dq8 = torch, dq8
        self.n = workloads.C3_NUMEL
        t0 = time.time()
        self.x, self.host = [], []
        for w in range(K_WORKERS):
            h = workloads.bucket(5, worker=w)
            self.x.append(torch.from_numpy(h).cuda())
            if keep_host:
                self.host.append(h)
        torch.cuda.synchronize()
        print("set-up: generated %d workers' buckets in %.1f s" % (K_WORKERS, time.time() - t0), file=sys.stderr, flush=True)
        n = self.n
        self.max_nb = (n + 3) // 4  # the shortest block of the sweep has four elements
        self.sets = []
        for r in range(N_SETS):
            self.sets.append({
                "x": self.x[r],
                "codes": [torch.empty(n, dtype=torch.uint8, device="cuda") for _ in range(K_WORKERS)],
                "scales_buf": [torch.empty(self.max_nb, dtype=torch.float32, device="cuda") for _ in range(K_WORKERS)],
                "amax": torch.empty(self.max_nb, dtype=torch.float32, device="cuda"),
                "c_out": torch.empty(n, dtype=torch.uint8, device="cuda"),
                "s_out": torch.empty(self.max_nb, dtype=torch.float32, device="cuda"),
                "dec": torch.empty(n, dtype=torch.float32, device="cuda"),
                "mean": torch.empty(n, dtype=torch.float32, device="cuda"),
                "rc": torch.empty(n, dtype=torch.uint8, device="cuda"),
                "rs": torch.empty(self.max_nb, dtype=torch.float32, device="cuda"),
            })
        self.block = None

    def prepare(self, kind, block):
        """Encodes the K workers with this block length into every set (set-up, not timed) and fills the means."""
        dq8, torch = self.dq8, self.torch
        self.block = block
        self.nb = dq8.n_blocks(self.n, block)
        for w in range(K_WORKERS):
            c0, s0 = self.sets[0]["codes"][w], self.sets[0]["scales_buf"][w]
            dq8.encode(kind, self.x[w], block, scales=s0, codes=c0)
            for st in self.sets[1:]:
                st["codes"][w].copy_(c0)
                st["scales_buf"][w][:self.nb].copy_(s0[:self.nb])
        self.block_len = self.n if (block == 0 or block > self.n) else block
        for r, st in enumerate(self.sets):
            st["codes"] = st["codes"][:K_WORKERS]
            st["scales"] = [s[:self.nb] for s in st["scales_buf"]]
            dq8.decode_accumulate_avg(kind, st["codes"], st["scales"], block, out=st["mean"])
            # as a step leaves it: s_out of set r holds the block maxima of the next set's x (error_stats reads them)
            dq8.encode(kind, self.sets[(r + 1) % N_SETS]["x"], block, scales=st["s_out"], codes=st["c_out"])
            st["stats"] = torch.empty((self.nb, 4), dtype=torch.float64, device="cuda")
            st["means"] = torch.empty(2, dtype=torch.float64, device="cuda")
        torch.cuda.synchronize()

    def step_calls(self, i, kind=KIND, K=K_WORKERS):
        """The five calls of step i.  See the module docstring for which set each call reads."""
        dq8, B = self.dq8, self.block
        s0, s1, s2 = self.sets[i % N_SETS], self.sets[(i + 1) % N_SETS], self.sets[(i + 2) % N_SETS]
        return [
            ("absmax", lambda: dq8.absmax(s0["x"], B, scales=s0["amax"])),
            ("encode", lambda: dq8.encode(kind, s1["x"], B, scales=s0["s_out"], codes=s0["c_out"])),
            ("decode", lambda: dq8.decode(kind, s0["codes"][0], s0["scales"][0], B, out=s0["dec"])),
            ("decode_accumulate_avg", lambda: dq8.decode_accumulate_avg(kind, s1["codes"][:K], s1["scales"][:K], B, out=s0["mean"])),
            # the mean written two steps earlier in the rotation (long evicted), not the one just produced
            ("re_encode", lambda: dq8.encode(kind, s2["mean"], B, scales=s0["rs"], codes=s0["rc"])),
        ]

    def extra_calls(self, i, kind=KIND, K=K_WORKERS):
        """Calls beside the step: timed per kernel only."""
        dq8, B = self.dq8, self.block
        st, nxt = self.sets[i % N_SETS], self.sets[(i + 1) % N_SETS]
        return [
            ("decode_avg_encode", lambda: dq8.decode_avg_encode(kind, st["codes"][:K], st["scales"][:K], B,
                                                                scales=st["rs"], codes=st["rc"])),
            ("decode_accumulate_avg_local", lambda: dq8.decode_accumulate_avg(kind, st["codes"][:K], st["scales"][:K], B,
                                                                              out=st["dec"], local=nxt["x"])),
            ("error_stats", lambda: dq8.error_stats(kind, nxt["x"], B, scales=st["s_out"], scales_given=True,
                                                    stats=st["stats"], means=st["means"])),
            ("decode_avg_encode_7_local", lambda: dq8.decode_avg_encode(kind, st["codes"][:7], st["scales"][:7], B,
                                                                        local=nxt["x"], scales=st["rs"], codes=st["rc"])),
            ("encode_mantissa", lambda: dq8.encode(dq8.MANTISSA, nxt["x"], B, scales=st["rs"], codes=st["rc"])),
        ]


def rates(alg_bytes, ms, n, copy_gbps):
    gbps = alg_bytes / (ms * 1e-3) / 1e9
    return {"ms": round(ms, 5), "fp32_GBps": round(4 * n / (ms * 1e-3) / 1e9, 1), "hbm_GBps": round(gbps, 1),
            "frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4), "frac_of_copy": round(gbps / copy_gbps, 4),
            "algorithmic_bytes": alg_bytes}


def run_default(args, torch, dq8, internal, workloads):
    bk = Bucket(torch, dq8, workloads, keep_host=not args.no_cpu_baseline)
    n = bk.n
    bk.prepare(KIND, BLOCK)
    nb = bk.nb

    def step(i):
        for _, f in bk.step_calls(i):
            f()

    # ---- clock settling (untimed): groups of ten steps until the last three groups agree within 1 %
    settle_groups, recent, settled_ms = 0, [], None
    it = 0
    while settle_groups < args.max_settle_groups:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            step(it)
            it += 1
        torch.cuda.synchronize()
        recent = (recent + [(time.perf_counter() - t0) / 10 * 1e3])[-3:]
        settle_groups += 1
        if len(recent) == 3 and max(recent) - min(recent) <= 0.01 * min(recent):
            settled_ms = recent[-1]
            break
    prev = recent[-1] if recent else None
    # ---- timed region: W warm-up steps, then exactly K steps between synchronisations
    for i in range(args.warmup):
        step(it + i)
    it += args.warmup
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(it + i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    value = 5 * 4 * n / (elapsed / args.steps) / 1e9

    # ---- calibration: plain copy with the same access pattern (context for the fractions below)
    copy_gbps = copy_rate_gbps(torch, internal, [s["x"] for s in bk.sets], [s["dec"] for s in bk.sets], n)

    # ---- per-kernel durations: one call at a time over the same rotating buffers
    def all_calls(i):
        return bk.step_calls(i) + bk.extra_calls(i)

    names = [nm for nm, _ in all_calls(0)]
    launches = max(args.steps, MIN_LAUNCHES)
    alg = algorithmic_bytes(n, nb)
    kernels = {}
    for idx, nm in enumerate(names):
        if args.only and nm != args.only:
            continue
        ms = event_time_ms(torch, lambda i, idx=idx: all_calls(i)[idx][1](), launches, prime=PRIME)
        kernels[nm] = rates(alg[nm], ms, n, copy_gbps)

    dom = "decode_accumulate_avg" if "decode_accumulate_avg" in kernels else list(kernels)[0]
    traffic = recorded_traffic(dom)
    roof = {"bound": "hbm", "kernel": dom, "achieved": kernels[dom]["hbm_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": kernels[dom]["frac_of_peak"], "frac_of_copy": kernels[dom]["frac_of_copy"], "traffic": traffic,
            "traffic_source": (TRAFFIC_PROFILE + " (rocprofv3 FETCH_SIZE / WRITE_SIZE of an earlier run, not this one)") if traffic else None,
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
        "kernel_timing": "median of %d groups of %d consecutive launches between HIP events" % (GROUPS, launches),
        "settle": {"steps": 10 * settle_groups, "settled": settled_ms is not None,
                   "last_ms_per_step": None if prev is None else round(settled_ms if settled_ms is not None else prev, 4)},
        "device": device_info(internal),
        "copy_kernel_GBps": round(copy_gbps, 1),
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(bk.host)
    print(json.dumps(out), flush=True)


# ------------------------------------------------------------------------------------------------ sweeps

SWEEP_BLOCKS = [0, 4, 64, 256, 512, 1000, 1024, 2048, 3000, 4096, 5000, 8192, 9216, 12288, 16384, 65536]
SWEEP_WORKERS = [1, 2, 3, 4, 5, 6, 7, 8, 16, 32]
SWEEP_LAUNCHES = 30


def sweep_line(**kw):
    print(json.dumps(kw), flush=True)


def sweep_bucket(what, torch, dq8, internal, workloads):
    """Every call on the 61 100 840-element bucket at other block lengths (K = 8) and other worker counts (block 4096)."""
    bk = Bucket(torch, dq8, workloads, keep_host=False)
    n = bk.n
    bk.prepare(KIND, BLOCK)
    for i in range(100):  # settle the clocks
        for _, f in bk.step_calls(i):
            f()
    torch.cuda.synchronize()
    copy_gbps = copy_rate_gbps(torch, internal, [s["x"] for s in bk.sets], [s["dec"] for s in bk.sets], n)
    sweep_line(sweep="calibration", copy_kernel_GBps=round(copy_gbps, 1), n=n, launches_per_group=SWEEP_LAUNCHES, groups=3)

    def timed(idx_name, calls_of, K, block_label, sweep):
        table = dict(algorithmic_bytes(n, bk.nb, K))
        for idx, nm in enumerate([nm for nm, _ in calls_of(0)]):
            if nm not in idx_name:
                continue
            try:
                ms = event_time_ms(torch, lambda i, idx=idx: calls_of(i)[idx][1](), SWEEP_LAUNCHES, groups=3, prime=PRIME)
            except dq8.Dq8Error as e:  # e.g. the one-call second round with a block too long to hold
                sweep_line(sweep=sweep, block=block_label, K=K, call=nm, error=str(e))
                continue
            alg = table[nm]
            if nm == "encode" and bk.block_len > 16384:
                alg += 4 * n  # a block too long to hold: the input is read twice
            sweep_line(sweep=sweep, block=block_label, K=K, call=nm, **rates(alg, ms, n, copy_gbps))

    if "blocks" in what:
        for block in SWEEP_BLOCKS:
            bk.prepare(KIND, block)
            timed({"absmax", "encode", "decode", "decode_accumulate_avg"}, bk.step_calls, K_WORKERS, block, "blocks")
            timed({"decode_avg_encode"}, bk.extra_calls, K_WORKERS, block, "blocks")
    if "workers" in what:
        bk.prepare(KIND, BLOCK)
        for st in bk.sets:  # 32 workers: the eight buffers of a set, and three more copies of them
            for rep in range(3):
                st["codes"] = st["codes"] + [c.clone() for c in st["codes"][:K_WORKERS]]
                st["scales"] = st["scales"] + [s.clone() for s in st["scales"][:K_WORKERS]]
        for K in SWEEP_WORKERS:
            timed({"decode_accumulate_avg"}, lambda i, K=K: bk.step_calls(i, K=K), K, BLOCK, "workers")
            timed({"decode_avg_encode"}, lambda i, K=K: bk.extra_calls(i, K=K), K, BLOCK, "workers")


def sweep_configs(torch, dq8, internal, workloads):
    """C1, C2 (one scale per tensor: block 0, one call per tensor) and C4 (one scale per row) as they would be used:
    encode every tensor, then decode every tensor.  Enough copies of a configuration to exceed 1 GB of buffers are
    walked in rotation, so no pass finds its data in a cache."""
    big = torch.empty(workloads.C3_NUMEL, dtype=torch.float32, device="cuda")
    big2 = torch.empty_like(big)
    copy_gbps = copy_rate_gbps(torch, internal, [big, big2], [big2, big], big.numel())
    del big, big2
    plans = [("C1", 1, [dq8.DYNAMIC_TREE], 0), ("C2", 2, [dq8.DYNAMIC_TREE, dq8.LINEAR, dq8.STATIC_TREE], 0),
             ("C4", 4, [dq8.DYNAMIC_TREE], 4096)]
    names = {dq8.DYNAMIC_TREE: "dynamic_tree", dq8.LINEAR: "linear", dq8.STATIC_TREE: "static_tree"}
    for label, config, kinds, block in plans:
        host = [t for _, t in workloads.tensors(config)]
        n_total = sum(t.size for t in host)
        copies = max(2, -(-(1 << 30) // (n_total * 9)))
        xs = [[torch.from_numpy(t).cuda() for t in host] for _ in range(copies)]
        cs = [[torch.empty(t.size, dtype=torch.uint8, device="cuda") for t in host] for _ in range(copies)]
        ss = [[torch.empty(dq8.n_blocks(t.size, block), dtype=torch.float32, device="cuda") for t in host] for _ in range(copies)]
        outs = [[torch.empty(t.size, dtype=torch.float32, device="cuda") for t in host] for _ in range(copies)]
        # a tensor whose single block is too long to hold is read twice by the compression
        enc_bytes = sum((9 if (block == 0 and t.size > 16384) else 5) * t.size + 4 * dq8.n_blocks(t.size, block) for t in host)
        dec_bytes = sum(5 * t.size + 4 * dq8.n_blocks(t.size, block) for t in host)
        for kind in kinds:
            def enc_pass(i):
                r = i % copies
                for x, c, s in zip(xs[r], cs[r], ss[r]):
                    dq8.encode(kind, x, block, scales=s, codes=c)

            def dec_pass(i):
                r = i % copies
                for c, s, o in zip(cs[r], ss[r], outs[r]):
                    dq8.decode(kind, c, s, block, out=o)

            for r in range(copies):
                enc_pass(r)
            torch.cuda.synchronize()
            launches = max(copies, 20)
            for call, f, alg in (("encode", enc_pass, enc_bytes), ("decode", dec_pass, dec_bytes)):
                ms = event_time_ms(torch, f, launches, groups=3)
                sweep_line(sweep="configs", config=label, kind=names[kind], call=call, launch="calls", tensors=len(host),
                           elements=n_total, block=block, copies=copies, calls_per_pass=len(host),
                           **rates(alg, ms, n_total, copy_gbps))
                # the same pass recorded once per copy as a HIP graph and replayed: one launch from the host per pass
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                graphs = []
                for r in range(copies):
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g, stream=side):
                        f(r)
                    graphs.append(g)
                torch.cuda.synchronize()
                ms = event_time_ms(torch, lambda i: graphs[i % copies].replay(), launches, groups=3)
                sweep_line(sweep="configs", config=label, kind=names[kind], call=call, launch="graph", tensors=len(host),
                           elements=n_total, block=block, copies=copies, calls_per_pass=len(host),
                           **rates(alg, ms, n_total, copy_gbps))
                del graphs
            if block == 0:
                # the whole configuration as one array with one scale per tensor: one call per pass
                bounds = torch.tensor([0] + list(itertools.accumulate(t.size for t in host)), dtype=torch.int64, device="cuda")
                fx = [torch.cat(x) for x in xs]
                fc = [torch.empty(n_total, dtype=torch.uint8, device="cuda") for _ in range(copies)]
                fs = [torch.empty(len(host), dtype=torch.float32, device="cuda") for _ in range(copies)]
                fo = [torch.empty(n_total, dtype=torch.float32, device="cuda") for _ in range(copies)]
                seg_enc = lambda i: dq8.encode_segments(kind, fx[i % copies], bounds, scales=fs[i % copies], codes=fc[i % copies])
                seg_dec = lambda i: dq8.decode_segments(kind, fc[i % copies], fs[i % copies], bounds, out=fo[i % copies])
                for r in range(copies):
                    seg_enc(r)
                torch.cuda.synchronize()
                seg_bytes = 4 * len(host)
                for call, f, alg in (("encode_segments", seg_enc, 9 * n_total + seg_bytes), ("decode_segments", seg_dec, 5 * n_total + seg_bytes)):
                    ms = event_time_ms(torch, f, launches, groups=3)
                    sweep_line(sweep="configs", config=label, kind=names[kind], call=call, launch="calls", tensors=len(host),
                               elements=n_total, block=block, copies=copies, calls_per_pass=1, **rates(alg, ms, n_total, copy_gbps))
                    side = torch.cuda.Stream()
                    side.wait_stream(torch.cuda.current_stream())
                    graphs = []
                    for r in range(copies):
                        g = torch.cuda.CUDAGraph()
                        with torch.cuda.graph(g, stream=side):
                            f(r)
                        graphs.append(g)
                    torch.cuda.synchronize()
                    ms = event_time_ms(torch, lambda i: graphs[i % copies].replay(), launches, groups=3)
                    sweep_line(sweep="configs", config=label, kind=names[kind], call=call, launch="graph", tensors=len(host),
                               elements=n_total, block=block, copies=copies, calls_per_pass=1, **rates(alg, ms, n_total, copy_gbps))
                    del graphs
                del fx, fc, fs, fo
            else:
                # rows of one length: the matrices back to back are one array with that block length, one call per pass
                fx = [torch.cat(x) for x in xs]
                fc = [torch.empty(n_total, dtype=torch.uint8, device="cuda") for _ in range(copies)]
                fs = [torch.empty(dq8.n_blocks(n_total, block), dtype=torch.float32, device="cuda") for _ in range(copies)]
                fo = [torch.empty(n_total, dtype=torch.float32, device="cuda") for _ in range(copies)]
                one_enc = lambda i: dq8.encode(kind, fx[i % copies], block, scales=fs[i % copies], codes=fc[i % copies])
                one_dec = lambda i: dq8.decode(kind, fc[i % copies], fs[i % copies], block, out=fo[i % copies])
                for r in range(copies):
                    one_enc(r)
                torch.cuda.synchronize()
                alg = 5 * n_total + 4 * dq8.n_blocks(n_total, block)
                for call, f in (("encode, one array", one_enc), ("decode, one array", one_dec)):
                    ms = event_time_ms(torch, f, launches, groups=3)
                    sweep_line(sweep="configs", config=label, kind=names[kind], call=call, launch="calls", tensors=len(host),
                               elements=n_total, block=block, copies=copies, calls_per_pass=1, **rates(alg, ms, n_total, copy_gbps))
                del fx, fc, fs, fo
        del xs, cs, ss, outs


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--max-settle-groups", type=int, default=60,
                    help="upper limit of the untimed clock-settling phase, in groups of ten steps (0: none, e.g. under a profiler)")
    ap.add_argument("--only", default=None, help="time only this call in the per-kernel pass (profiling aid)")
    ap.add_argument("--sweep", nargs="?", const="blocks,workers,configs", default=None,
                    help="print one JSON line per (block length | worker count | small configuration) instead of the bench line")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_1511_04561_amd import _internal as internal
    from paper_1511_04561_amd import dq8, workloads

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    dq8.init()
    if args.sweep is not None:
        what = set(args.sweep.split(","))
        if what & {"blocks", "workers"}:
            sweep_bucket(what, torch, dq8, internal, workloads)
        if "configs" in what:
            sweep_configs(torch, dq8, internal, workloads)
        return
    run_default(args, torch, dq8, internal, workloads)


if __name__ == "__main__":
    main()
