#!/usr/bin/env python3
"""Benchmark of the truncated-quantization hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic gradients of a
benchmark configuration (default: config 2, 11.2 M fp32 elements x 8 workers, uniform
grid): for each simulated worker tq_stats -> tq_params -> tq_compress, then one fused
tq_decompress_aggregate over the N payloads.  Inputs are resident in HBM before timing.

Prints ONE JSON line.  `value` is GB/s of gradient input over the whole step (all four
entry points); `compress_decode_gbps` is the same input over the compress + decode kernels
only, the narrower quantity the headline metric names.  `roofline` is for the dominant
kernel (tq_compress_kernel), its duration measured with HIP events on the launch stream;
`cpu_baseline` is the scalar oracle timed on this host on the same inputs.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--bits", type=int, default=0, help="0 = the workload's first b")
    ap.add_argument("--grid", type=int, default=-1, help="-1 = the workload's first grid")
    ap.add_argument("--launch", default="batched", choices=["batched", "per-worker", "streams"],
                    help="how the N simulated workers are launched (see Path.step)")
    ap.add_argument("--buffer-sets", type=int, default=2,
                    help="different input gradients per worker, used in turn (1 = the same buffers every step)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="profiling aid: only run device-to-device copies of 1 GiB, the known-size "
                         "kernel that scales the FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--kernel-only", default="", help="profiling aid: loop one entry point only "
                    "(stats|params|compress|decode)")
    return ap.parse_args()


class Path:
    """Device buffers of one workload and the launch sequence of one step."""

    def __init__(self, wl, bits, grid, mode="batched", sets=2):
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

    def stats_i(self, i):
        self.B.tq_stats(self.g[i], self.stats[i], self.ws[i], self.be, self.wl.g_min)

    def params_i(self, i):
        self.B.tq_params(self.stats[i], self.params[i], self.bits, self.grid)

    def compress_i(self, i):
        self.B.tq_compress(self.g[i], self.params[i], self.pay[i], self.bits, 0x5EED, i, self.step_no, self.be)

    def decode(self):
        self.B.tq_decompress_aggregate(self.pay, self.params, self.out, self.bits, self.be)

    def stats_all(self):
        self.B.tq_stats_multi(self.g, self.stats, self.ws_all, self.be, self.wl.g_min)

    def params_all(self):
        self.B.tq_params_multi(self.stats, self.params, self.bits, self.grid)

    def compress_all(self):
        self.B.tq_compress_multi(self.g, self.params, self.pay, self.bits, 0x5EED, 0, self.step_no, self.be)

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
        """Same launches on one stream, each bracketed by events on the launch stream.
        rec[name] collects (start, end, launches covered)."""
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


def cpu_baseline(path):
    """The oracle, as it stands, on the same inputs: one whole step on one host thread."""
    from oracle import binding as O
    from oracle import params as OP
    from paper_2402_01798_amd import synth
    N, d, be, bits = path.N, path.d, path.be, path.bits
    # bounded sample: at most ~1e8 element-encodes (about 5 s of scalar work per 1e8)
    n_workers = max(1, min(N, int(1.0e8 // d)))
    d_s = d if d <= 100_000_000 else (100_000_000 >> 20) << 20
    gs = [synth.as_numpy(path.g[i][:d_s]) for i in range(n_workers)]
    t0 = time.perf_counter()
    pays, Ps = [], []
    for i in range(n_workers):
        S = O.stats(gs[i], bucket_elems=be, g_min=path.wl.g_min)
        P = OP.tq_params(S, bits, path.grid)
        pays.append(O.compress(gs[i], P, 0x5EED, i, 0, bucket_elems=be))
        Ps.append(P)
    O.decompress_aggregate(pays, Ps, d_s, bits, bucket_elems=be)
    dt = time.perf_counter() - t0
    nbytes = n_workers * d_s * path.g[0].element_size()
    return {"value": nbytes / dt / 1e9, "unit": "GB/s of gradient input", "cores": 1, "kind": "oracle",
            "sample": "%d of %d workers x %d of %d elements, whole step (stats, params, compress, "
                      "decode-aggregate), %.1f s" % (n_workers, N, d_s, d, dt)}


def load_traffic(kernel, workload, bits):
    """HBM bytes per launch from committed rocprofv3 --pmc summaries, if any (data, not code)."""
    p = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        table = json.load(open(p))
        return table.get("%s/%s/b%d" % (kernel, workload, bits))
    except (OSError, ValueError):
        return None


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
    path = Path(wl, bits, grid, a.launch, max(1, a.buffer_sets))
    torch.cuda.synchronize()

    if a.kernel_only:
        # profiling aid: the named entry point alone (after one full step so its inputs exist)
        path.step()
        if a.launch == "batched":
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

    for _ in range(a.warmup):
        path.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        path.step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / a.steps * 1e3

    # per-kernel durations: the same K steps again, every launch bracketed by HIP events
    rec = {"stats": [], "params": [], "compress": [], "decode": []}
    for _ in range(a.steps):
        path.step_instrumented(rec)
    torch.cuda.synchronize()
    # microseconds per STEP spent in each entry point (all N workers)
    avg_us = {k: sum(s.elapsed_time(e) for s, e in v) / a.steps * 1e3 for k, v in rec.items()}

    # the compress launch on its own, its input NOT left in the memory-side cache by a
    # statistics pass just before it: reading 1 GiB of other data evicts the cache (and leaves
    # no dirty lines behind) before every launch
    cold_us = None
    if a.launch == "batched":
        flush = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        pairs = []
        for k in range(a.steps):
            path.g = path.gsets[k % len(path.gsets)]
            flush.sum()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); path.compress_all(); e1.record()
            pairs.append((e0, e1))
        torch.cuda.synchronize()
        cold_us = sum(s_.elapsed_time(e_) for s_, e_ in pairs) / a.steps * 1e3
        del flush

    in_bytes = path.input_bytes()
    value = in_bytes / (ms_per_step * 1e-3) / 1e9
    cd_us = avg_us["compress"] + avg_us["decode"]
    cd_gbps = in_bytes / (cd_us * 1e-6) / 1e9
    cd_bytes = path.N * path.bytes_compress() + path.bytes_decode()
    step_bytes = cd_bytes + path.N * path.bytes_stats()
    comp_gbps = path.N * path.bytes_compress() / (avg_us["compress"] * 1e-6) / 1e9

    out = {
        "metric": "compress+decode-aggregate GB/s of fp32 gradient input; fraction of HBM peak",
        "value": round(value, 1),
        "unit": "GB/s of gradient input (whole step: stats+params+compress x N, decode-aggregate)",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if wl.dtype == torch.float32 else "bf16->f32",
        "data": "synthetic (seeded symmetric power-law gradients; recipe in paper_2402_01798_amd/synth.py)",
        "config": {"workload": "%s: d=%d x N=%d workers, %s, b=%d, %s grid, bucket_elems=%d" % (
                       wl.name, wl.d, wl.workers, "fp32" if wl.dtype == torch.float32 else "bf16", bits,
                       "uniform" if grid == 0 else "non-uniform", wl.bucket_elems),
                   "bits": bits, "grid": grid, "workers": wl.workers, "d": wl.d},
        "hbm_frac_whole_step": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "compress_decode_gbps": round(cd_gbps, 1),
        "compress_decode_hbm_frac": round(cd_bytes / (cd_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
        "launch": a.launch,
        "buffer_sets": len(path.gsets),
        "stage_us_per_step": {k: round(v, 2) for k, v in avg_us.items()},
        "stage_gbps": {"stats": round(path.N * path.bytes_stats() / avg_us["stats"] / 1e3, 1),
                        "compress": round(comp_gbps, 1),
                        "decode": round(path.bytes_decode() / avg_us["decode"] / 1e3, 1)},
        "compress_cold": None if cold_us is None else {
            "us": round(cold_us, 2), "gbps": round(path.N * path.bytes_compress() / cold_us / 1e3, 1),
            "note": "same launch with the memory-side cache evicted first; in the step the statistics "
                    "pass has just read the same gradients and part of them is still cached"},
        "roofline": {"kernel": "tq_compress_kernel", "bound": "hbm", "achieved": round(comp_gbps, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(comp_gbps / HBM_PEAK_GBPS, 4),
                     "traffic": load_traffic("tq_compress_kernel", wl.name, bits)},
    }
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(path)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
