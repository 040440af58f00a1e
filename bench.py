#!/usr/bin/env python3
"""Benchmark of the truncated-quantization hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic gradients of a benchmark
configuration: tq_stats -> tq_params -> tq_compress for the N simulated workers (one batched
launch each), then one fused tq_decompress_aggregate over the N payloads.  Inputs are resident
in HBM before timing.

The headline workload (`value`, `config`, `roofline`) is configuration 4, the largest fp32
one: 8 workers x 124 M elements, uniform 2-bit codebook, buckets of 2^20 -- 4 GB of gradients
per step, so nothing a kernel reads was left in the 256 MB memory-side cache by the kernel
before it.  The same run then times every other variant the benchmark plan names (config 2 at
b = 2 and b = 4, config 3, config 4 with the non-uniform codebook, config 5) with fewer steps
and reports them under `configs`.

Prints ONE JSON line.  `value` is GB/s of gradient input over the whole step (all four entry
points); `compress_decode_gbps` is the same input over the compress + decode launches only,
the narrower quantity the headline metric names.  `roofline` is for the compress kernel, the
longest kernel of that pair, its duration measured with HIP events on the launch stream inside
the timed steps; `cpu_baseline` is the scalar oracle timed on this host's cores on a sample of
the same inputs.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published peak
# Vector-ALU ceiling for kernels bound by instruction issue: 256 compute units x 4 SIMDs x 16
# lanes x 2.4 GHz = 39.3 T lane-operations/s (one fp32 or int32 operation per lane and cycle;
# the published 157.3 TFLOP/s counts packed two-wide fused multiply-adds, which this build
# does not use).
ALU_PEAK_TLOPS = 256 * 4 * 16 * 2.4e9 / 1e12

# (workload, bits, grid) of every variant the benchmark plan names; the first is the headline
VARIANTS = [("cfg4", 2, 0), ("cfg4", 2, 1), ("cfg2", 2, 0), ("cfg2", 4, 0), ("cfg3", 3, 1), ("cfg5", 2, 1)]

# vector-ALU lane-operations per element of the compress kernel's variants, as rocprofv3's
# SQ_INSTS_VALU counts them (profiles/valu_instructions.txt): they decide which ceiling binds
COMPRESS_VALU_PER_ELEM = {"f32/b2/g0": 15.5, "f32/b2/g1": 20.2, "f32/b4/g0": 20.2, "f32/b3/g1": 29.4,
                          "bf16/b2/g1": 20.5}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg4", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--bits", type=int, default=0, help="0 = the workload's first b")
    ap.add_argument("--grid", type=int, default=-1, help="-1 = the workload's first grid")
    ap.add_argument("--launch", default="batched", choices=["batched", "per-worker", "streams"],
                    help="how the N simulated workers are launched (see Path.step)")
    ap.add_argument("--buffer-sets", type=int, default=2,
                    help="different input gradients per worker, used in turn (1 = the same buffers every step)")
    ap.add_argument("--other-configs", default="all", choices=["all", "none"],
                    help="also time the other variants of the benchmark plan (reported under `configs`)")
    ap.add_argument("--other-steps", type=int, default=20, help="timed steps of each other variant")
    ap.add_argument("--segments", action="store_true",
                    help="one record per layer of the workload's recipe (the *_segments entry points)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="profiling aid: only run device-to-device copies of 1 GiB, the known-size "
                         "kernel that scales the FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--kernel-only", default="", help="profiling aid: loop one entry point only "
                    "(stats|params|compress|decode)")
    return ap.parse_args()


class Path:
    """Device buffers of one workload and the launch sequence of one step."""

    def __init__(self, wl, bits, grid, mode="batched", sets=2, segments=False):
        import torch
        from paper_2402_01798_amd import binding as B
        from paper_2402_01798_amd import synth
        self.B, self.torch = B, torch
        self.wl, self.bits, self.grid = wl, bits, grid
        self.N, self.d, self.be = wl.workers, wl.d, wl.bucket_elems
        # `sets` different gradients per worker, used in turn: a step never finds the gradient it
        # reads left in the memory-side cache by the step before (in training every step's
        # gradient is new)
        self.gsets = [[synth.make_gradient(wl, i + 64 * s, "cuda") for i in range(self.N)] for s in range(sets)]
        self.g = self.gsets[0]
        self.stats = [B.alloc_stats(self.d, self.be) for _ in range(self.N)]
        # one statistics workspace per simulated worker: their chains run on separate streams
        self.ws = [B.alloc_stats_workspace(self.d, self.be) for _ in range(self.N)]
        self.ws_all = torch.empty(self.N * B.stats_workspace_bytes(self.d, self.be), dtype=torch.uint8,
                                  device="cuda")
        self.mode = mode
        self.streams = [torch.cuda.Stream() for _ in range(self.N)] if mode == "streams" else None
        self.done = [torch.cuda.Event() for _ in range(self.N)]
        self.start = torch.cuda.Event()
        self.params = [B.alloc_params(self.d, self.be) for _ in range(self.N)]
        self.pay = [B.alloc_payload(self.d, bits) for _ in range(self.N)]
        self.out = torch.empty(self.d, dtype=torch.float32, device="cuda")
        self.step_no = 0
        # per-layer quantization: one record per layer of the workload's recipe instead of per bucket,
        # through the *_segments entry points
        self.seg = None
        if segments:
            self.seg = B.Segments(synth.layer_segments(wl, self.d))
            self.stats = [torch.empty(self.seg.nseg * B.STATS_BYTES, dtype=torch.uint8, device="cuda") for _ in range(self.N)]
            self.params = [torch.empty(self.seg.nseg * B.PARAMS_BYTES, dtype=torch.uint8, device="cuda") for _ in range(self.N)]
            self.ws_all = torch.empty(self.N * B.stats_segments_workspace_bytes(self.d, self.seg.nseg), dtype=torch.uint8,
                                      device="cuda")
            self.ws = [self.ws_all] * self.N             # one stream: the per-worker launches run in turn
            if mode == "streams":
                raise SystemExit("--segments runs batched or per-worker")

    def describe(self):
        torch = self.torch
        what = "bucket_elems=%d" % self.be if self.seg is None else "%d layer segments" % self.seg.nseg
        return "%s: d=%d x N=%d workers, %s, b=%d, %s grid, %s" % (
            self.wl.name, self.d, self.N, "fp32" if self.wl.dtype == torch.float32 else "bf16", self.bits,
            "uniform" if self.grid == 0 else "non-uniform", what)

    def stats_i(self, i):
        if self.seg is not None:
            return self.B.tq_stats_segments(self.g[i], self.seg, self.stats[i], self.ws[i], self.wl.g_min)
        self.B.tq_stats(self.g[i], self.stats[i], self.ws[i], self.be, self.wl.g_min)

    def params_i(self, i):
        self.B.tq_params(self.stats[i], self.params[i], self.bits, self.grid)

    def compress_i(self, i):
        if self.seg is not None:
            return self.B.tq_compress_segments(self.g[i], self.seg, self.params[i], self.pay[i], self.bits, 0x5EED, i,
                                               self.step_no)
        self.B.tq_compress(self.g[i], self.params[i], self.pay[i], self.bits, 0x5EED, i, self.step_no, self.be, self.grid)

    def decode(self):
        if self.seg is not None:
            return self.B.tq_decompress_aggregate_segments(self.pay, self.params, self.seg, self.out, self.bits)
        self.B.tq_decompress_aggregate(self.pay, self.params, self.out, self.bits, self.be)

    def stats_all(self):
        if self.seg is not None:
            return self.B.tq_stats_segments_multi(self.g, self.seg, self.stats, self.ws_all, self.wl.g_min)
        self.B.tq_stats_multi(self.g, self.stats, self.ws_all, self.be, self.wl.g_min)

    def params_all(self):
        self.B.tq_params_multi(self.stats, self.params, self.bits, self.grid)

    def compress_all(self):
        if self.seg is not None:
            return self.B.tq_compress_segments_multi(self.g, self.seg, self.params, self.pay, self.bits, 0x5EED, 0,
                                                     self.step_no)
        self.B.tq_compress_multi(self.g, self.params, self.pay, self.bits, 0x5EED, 0, self.step_no, self.be, self.grid)

    def step(self):
        """One pass of the whole path over all N simulated workers.

        batched (default): the N workers' statistics, parameters and compression each run as one
        launch (tq_*_multi), then one fused decode.  per-worker: one launch per worker and
        entry point on one stream.  streams: as per-worker, each worker's stats -> params ->
        compress chain on its own HIP stream, the decode waiting for all of them."""
        torch = self.torch
        self.g = self.gsets[self.step_no % len(self.gsets)]
        if self.mode == "batched":
            self.stats_all()
            self.params_all()
            self.compress_all()
        elif self.streams is None:
            for i in range(self.N):
                self.stats_i(i)
                self.params_i(i)
                self.compress_i(i)
        else:
            main = torch.cuda.current_stream()
            self.start.record(main)
            for i, st in enumerate(self.streams):
                st.wait_event(self.start)
                with torch.cuda.stream(st):
                    self.stats_i(i)
                    self.params_i(i)
                    self.compress_i(i)
                    self.done[i].record(st)
            for i in range(self.N):
                main.wait_event(self.done[i])
        self.decode()
        self.step_no += 1

    def step_instrumented(self, rec):
        """Same launches on one stream, each bracketed by events on the launch stream (the
        binding launches on torch's current stream, which is where these events are recorded).
        rec[name] collects (start, end)."""
        ev = lambda: self.torch.cuda.Event(enable_timing=True)
        self.g = self.gsets[self.step_no % len(self.gsets)]
        if self.mode == "batched":
            for name, fn in (("stats", self.stats_all), ("params", self.params_all), ("compress", self.compress_all)):
                a, b = ev(), ev()
                a.record(); fn(); b.record()
                rec[name].append((a, b))
        else:
            for i in range(self.N):
                for name, fn in (("stats", self.stats_i), ("params", self.params_i), ("compress", self.compress_i)):
                    a, b = ev(), ev()
                    a.record(); fn(i); b.record()
                    rec[name].append((a, b))
        a, b = ev(), ev()
        a.record(); self.decode(); b.record()
        rec["decode"].append((a, b))
        self.step_no += 1

    # algorithmic bytes (what the method itself must move), per launch of each kernel
    def bytes_stats(self):
        return self.d * self.g[0].element_size()

    def bytes_compress(self):
        return self.d * self.g[0].element_size() + self.d * self.bits / 8.0

    def bytes_decode(self):
        return self.d * (self.N * self.bits / 8.0 + 4.0)

    def input_bytes(self):
        return self.N * self.d * self.g[0].element_size()


def measure(path, steps, warmup, cold_steps):
    """Wall time of `steps` whole steps, then per-entry-point durations from HIP events on the
    launch stream over the same number of steps, then compress and decode launched alone with
    the memory-side cache evicted before each (reading 1 GiB of other data leaves it full of
    clean lines that are not this launch's input)."""
    torch = path.torch
    for _ in range(warmup):
        path.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        path.step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / steps * 1e3

    rec = {"stats": [], "params": [], "compress": [], "decode": []}
    for _ in range(steps):
        path.step_instrumented(rec)
    torch.cuda.synchronize()
    avg_us = {k: sum(s.elapsed_time(e) for s, e in v) / steps * 1e3 for k, v in rec.items()}

    cold = None
    if path.mode == "batched" and cold_steps > 0:
        flush = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        pairs = {"compress": [], "decode": []}
        for k in range(cold_steps):
            path.g = path.gsets[k % len(path.gsets)]
            for name, fn in (("compress", path.compress_all), ("decode", path.decode)):
                flush.sum()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(); fn(); e1.record()
                pairs[name].append((e0, e1))
        torch.cuda.synchronize()
        cold = {k: sum(s_.elapsed_time(e_) for s_, e_ in v) / cold_steps * 1e3 for k, v in pairs.items()}
        del flush

    N = path.N
    in_bytes = path.input_bytes()
    cd_bytes = N * path.bytes_compress() + path.bytes_decode()
    cd_us = avg_us["compress"] + avg_us["decode"]
    res = {
        "workload": path.describe(),
        "ms_per_step": round(ms_per_step, 4),
        "input_gbps_whole_step": round(in_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "hbm_frac_whole_step": round((cd_bytes + N * path.bytes_stats()) / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "stage_us_per_step": {k: round(v, 2) for k, v in avg_us.items()},
        "stage_gbps": {"stats": round(N * path.bytes_stats() / avg_us["stats"] / 1e3, 1),
                        "compress": round(N * path.bytes_compress() / avg_us["compress"] / 1e3, 1),
                        "decode": round(path.bytes_decode() / avg_us["decode"] / 1e3, 1)},
        "compress_decode_gbps": round(in_bytes / (cd_us * 1e-6) / 1e9, 1),
        "compress_decode_hbm_frac": round(cd_bytes / (cd_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
        "compress_melem_per_us": round(N * path.d / avg_us["compress"] / 1e6, 4),
    }
    if cold is not None:
        res["cold"] = {
            "compress_us": round(cold["compress"], 2), "decode_us": round(cold["decode"], 2),
            "compress_gbps": round(N * path.bytes_compress() / cold["compress"] / 1e3, 1),
            "compress_decode_hbm_frac": round(cd_bytes / ((cold["compress"] + cold["decode"]) * 1e-6) / 1e9
                                              / HBM_PEAK_GBPS, 4),
            "note": "each launch alone, the memory-side cache evicted first (1 GiB of other data read)"}
    return res


def cpu_baseline(path):
    """The oracle, as it stands, on a bounded sample of the same inputs: one whole step
    (statistics, parameters, compress for each worker, then the aggregate), its element loops
    spread over every host core this process may use."""
    from oracle import binding as O
    from oracle import params as OP
    from paper_2402_01798_amd import synth
    N, d, be, bits = path.N, path.d, path.be, path.bits
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    cores = max(1, min(cores, int(os.environ.get("OMP_NUM_THREADS", cores))))
    # bounded sample: about 2.5e8 element-encodes (10-30 core-seconds of scalar work)
    n_workers = max(1, min(N, int(2.5e8 // d)))
    d_s = d if d <= 250_000_000 else (250_000_000 >> 20) << 20
    gs = [synth.as_numpy(path.g[i][:d_s]) for i in range(n_workers)]
    t0 = time.perf_counter()
    pays, Ps = [], []
    for i in range(n_workers):
        S = O.stats(gs[i], bucket_elems=be, g_min=path.wl.g_min, threads=cores)
        P = OP.tq_params(S, bits, path.grid)
        pays.append(O.compress(gs[i], P, 0x5EED, i, 0, bucket_elems=be, threads=cores))
        Ps.append(P)
    O.decompress_aggregate(pays, Ps, d_s, bits, bucket_elems=be, threads=cores)
    dt = time.perf_counter() - t0
    nbytes = n_workers * d_s * path.g[0].element_size()
    return {"value": round(nbytes / dt / 1e9, 4), "unit": "GB/s of gradient input", "cores": cores, "kind": "oracle",
            "sample": "%d of %d workers x %d of %d elements, whole step (stats, params, compress, "
                      "decode-aggregate), %.1f s wall on %d threads" % (n_workers, N, d_s, d, dt, cores)}


def load_traffic(kernel, workload, bits, grid):
    """HBM bytes per launch from committed rocprofv3 --pmc summaries, if any (data, not code)."""
    p = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        table = json.load(open(p))
        return table.get("%s/%s/b%d/g%d" % (kernel, workload, bits, grid))
    except (OSError, ValueError):
        return None


def compress_roofline(path, res):
    """Roofline object of the compress kernel for one measured variant.  The kernel streams
    sz + b/8 bytes per element; whether HBM or the vector ALU binds depends on the variant's
    instruction count per element: the ALU needs valu/39.3T seconds per element at best, HBM
    (sz + b/8)/8T."""
    N = path.N
    comp_us = res["stage_us_per_step"]["compress"]
    gbps = N * path.bytes_compress() / comp_us / 1e3
    roof = {"kernel": "tq_compress_kernel", "bound": "hbm", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": round(gbps / HBM_PEAK_GBPS, 4),
            "traffic": load_traffic("tq_compress_kernel", path.wl.name, path.bits, path.grid)}
    key = "%s/b%d/g%d" % ("bf16" if path.g[0].element_size() == 2 else "f32", path.bits, min(path.grid, 1))
    valu = COMPRESS_VALU_PER_ELEM.get(key)
    if valu:
        t_alu = valu / (ALU_PEAK_TLOPS * 1e12)
        t_hbm = (path.bytes_compress() / path.d) / (HBM_PEAK_GBPS * 1e9)
        roof["valu_ops_per_elem"] = valu
        if t_alu > t_hbm:
            tlops = N * path.d * valu / (comp_us * 1e-6) / 1e12
            roof.update({"bound": "alu", "achieved": round(tlops, 2), "peak": round(ALU_PEAK_TLOPS, 1),
                         "unit": "T lane-op/s", "frac": round(tlops / ALU_PEAK_TLOPS, 4),
                         "hbm_frac": round(gbps / HBM_PEAK_GBPS, 4),
                         "note": "peak = one vector instruction per SIMD and cycle; this part overlaps "
                                 "instructions of different kinds (a mixed probe issues 41.3 T/s), so a "
                                 "kernel with no idle issue slot can read slightly above 1"})
    return roof


# vector-ALU lane-operations per element of the statistics kernel (profiles/valu_instructions.txt)
STATS_VALU_PER_ELEM = {"f32": 5.3, "f32/tail": 10.9, "bf16/tail": 9.9}


def stats_roofline(path, res):
    """Roofline object of the statistics kernel (the other long kernel of the step: it reads every
    gradient once, sz bytes per element, and writes a few MB of histograms)."""
    us = res["stage_us_per_step"]["stats"]
    sz = path.g[0].element_size()
    gbps = path.N * path.d * sz / us / 1e3
    kernel = "tq_stats_segments_partial_kernel" if path.seg is not None else "tq_stats_balanced_kernel"
    roof = {"kernel": kernel, "bound": "hbm", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(gbps / HBM_PEAK_GBPS, 4),
            "traffic": load_traffic("tq_stats_balanced_kernel", path.wl.name, path.bits, path.grid),
            "note": "duration of the statistics stage (both its kernels)"}
    valu = STATS_VALU_PER_ELEM.get(("bf16" if sz == 2 else "f32") + ("/tail" if path.wl.g_min > 0 else ""))
    if valu:
        roof["valu_ops_per_elem"] = valu
        roof["alu_frac"] = round(path.N * path.d * valu / (us * 1e-6) / 1e12 / ALU_PEAK_TLOPS, 4)
    return roof


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives); --gpus %d is not supported. "
              "Each GPU would be one worker, the aggregation one all-to-all of the packed codes." % a.gpus,
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2402_01798_amd import synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if a.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(a.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_each_way": src.numel() * 4, "copies": a.steps}))
        return
    wl = synth.WORKLOADS[a.workload]
    bits = a.bits or wl.bits[0]
    grid = a.grid if a.grid >= 0 else wl.grids[0]
    path = Path(wl, bits, grid, a.launch, max(1, a.buffer_sets), segments=a.segments)
    torch.cuda.synchronize()

    if a.kernel_only:
        # profiling aid: the named entry point alone (after one full step so its inputs exist)
        path.step()
        if path.mode == "batched":
            fn = {"stats": path.stats_all, "params": path.params_all, "compress": path.compress_all,
                  "decode": path.decode}[a.kernel_only]
        else:
            fn = {"stats": lambda: path.stats_i(0), "params": lambda: path.params_i(0),
                  "compress": lambda: path.compress_i(0), "decode": path.decode}[a.kernel_only]
        for _ in range(a.warmup + a.steps):
            fn()
        torch.cuda.synchronize()
        print(json.dumps({"kernel_only": a.kernel_only, "launches": a.warmup + a.steps}))
        return

    res = measure(path, a.steps, a.warmup, min(a.steps, 20))
    out = {
        "metric": "compress+decode-aggregate GB/s of fp32 gradient input; fraction of HBM peak",
        "value": res["input_gbps_whole_step"],
        "unit": "GB/s of gradient input (whole step: stats+params+compress x N, decode-aggregate)",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if wl.dtype == torch.float32 else "bf16->f32",
        "data": "synthetic (seeded symmetric power-law gradients; recipe in paper_2402_01798_amd/synth.py)",
        "config": {"workload": path.describe(), "bits": bits, "grid": grid, "workers": wl.workers, "d": wl.d},
        "hbm_frac_whole_step": res["hbm_frac_whole_step"],
        "compress_decode_gbps": res["compress_decode_gbps"],
        "compress_decode_hbm_frac": res["compress_decode_hbm_frac"],
        "launch": a.launch,
        "buffer_sets": len(path.gsets),
        "stage_us_per_step": res["stage_us_per_step"],
        "stage_gbps": res["stage_gbps"],
        "cold": res.get("cold"),
        "roofline": compress_roofline(path, res),
        "roofline_stats": stats_roofline(path, res),
    }
    if not a.no_cpu_baseline and not a.segments:
        out["cpu_baseline"] = cpu_baseline(path)

    if a.other_configs == "all" and a.launch == "batched":
        # every other variant of the benchmark plan, same method, fewer steps
        others = {}
        head = (a.workload, bits, grid)
        del path
        torch.cuda.empty_cache()
        for name, b, g in VARIANTS:
            if (name, b, g) == head:
                continue
            p2 = Path(synth.WORKLOADS[name], b, g, "batched", max(1, a.buffer_sets))
            torch.cuda.synchronize()
            r = measure(p2, a.other_steps, 3, min(a.other_steps, 10))
            r["roofline"] = compress_roofline(p2, r)
            r["roofline_stats"] = stats_roofline(p2, r)
            others["%s/b%d/%s" % (name, b, "uniform" if g == 0 else "nonuniform")] = r
            del p2
            torch.cuda.empty_cache()
        # config 4 once more with one record per LAYER of its recipe (variable-size segments)
        p2 = Path(synth.WORKLOADS["cfg4"], 2, 0, "batched", max(1, a.buffer_sets), segments=True)
        torch.cuda.synchronize()
        r = measure(p2, a.other_steps, 3, 0)
        r["roofline"] = compress_roofline(p2, r)
        r["roofline"]["kernel"] = "tq_compress_segments_kernel"
        r["roofline_stats"] = stats_roofline(p2, r)
        others["cfg4/b2/uniform/layer-segments"] = r
        del p2
        torch.cuda.empty_cache()
        out["configs"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
