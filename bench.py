#!/usr/bin/env python3
"""Benchmark of the RazorAttention hot path on one MI355X.

Workload of the top-level figures (default): benchmark configuration 3 -- a Llama-3-8B-shaped GQA
layer, batch 4, 32 query heads over 8 KV heads, head_dim 128, context 131072, bf16, 2 of 8 KV
heads retrieval, window max(4096, 15 % of context) + 4 sinks + compensation token.  Seeded
synthetic data.

A step is one razor_decode_attn call (append one token to every head, attend, combine) on a
cache that razor_compress built before the timed region.  `value` is the algorithmic HBM bytes of
a step divided by its wall time.  Also reported: per-step GPU time as median / min over HIP event
pairs, the same kernels on the uncompressed cache (every head marked retrieval), the compression
pass (repeated on warm buffers, and one-shot right after K and V were written), the dominant
kernel's own duration (HIP events around it on its stream) against the 8 TB/s roofline, the read
stream the device gives a kernel that only loads, and the fp64 CPU oracle timed on the host
cores.  `other_configs` carries the same measurements for configurations 1, 2, 4 and, memory
permitting, a few steps of configuration 5 (the 32-layer stack).

Other modes: --config N (N = 1..5 as the top-level workload), --head-scores, --wave-timeline
(per-wave finish times from the debug build), --read-stream-sweep and --read-after-write (the
memory-system tables kept under profiles/).

Prints one JSON line.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
METRIC = "compressed decode-attention HBM GB/s (% of peak) + speedup vs full cache, 128K"


def algorithmic_bytes_decode(desc, p_d, esize, B, Hq, out_esize=4, use_comp=True):
    """Bytes a decode step has to move: every cached K and V row once, the fp32 compensation
    tokens, Q in and O out.  Split-K partials are overhead, not counted."""
    rows = int(desc["rows"].astype("int64").sum())
    n_comp = int((desc["n_dropped"] > 0).sum()) if use_comp else 0
    return rows * 2 * p_d * esize + n_comp * 2 * p_d * 4 + B * Hq * p_d * esize + B * Hq * p_d * out_esize \
        + desc.size * desc.itemsize


def algorithmic_bytes_compress(desc, seq_lens, Hkv, p_d, esize):
    """Read every valid source row once, write every kept row once, plus the compensation tokens."""
    src_rows = int(seq_lens.astype("int64").sum()) * Hkv
    kept = int(desc["rows"].astype("int64").sum())
    return (src_rows + kept) * 2 * p_d * esize + desc.size * 2 * p_d * 4


def committed_traffic(config):
    """HBM bytes per launch of the dominant kernel as the committed rocprofv3 counter summary under
    profiles/ has them (FETCH_SIZE + WRITE_SIZE, scaled by a known-size copy): a figure from an
    earlier profiler run of this command, not a measurement of this run.  (bytes, file) or (None, None)."""
    name = f"decode_config{config}_hbm_traffic.txt"
    try:
        with open(os.path.join(ROOT, "profiles", name)) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return int(line.split(":")[1]), "profiles/" + name
    except OSError:
        pass
    return None, None


class HipEvents:
    """Raw HIP events (torch.cuda.Event only sees torch's notion of the stream)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self):
        ev = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(ev))
        assert rc == 0, f"hipEventCreate failed: {rc}"
        return ev

    def destroy(self, *evs):
        for e in evs:
            self.hip.hipEventDestroy(e)

    def record(self, ev, stream):
        assert self.hip.hipEventRecord(ev, ctypes.c_void_p(stream)) == 0

    def elapsed_ms(self, a, b):
        ms = ctypes.c_float()
        assert self.hip.hipEventSynchronize(b) == 0
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        assert rc == 0, f"hipEventElapsedTime failed: {rc}"
        return ms.value


def stats_us(ms_list):
    import numpy as np
    a = np.asarray(ms_list, dtype=np.float64) * 1e3
    return {"median": float(np.median(a)), "min": float(a.min()), "mean": float(a.mean()), "n": int(a.size)}


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


# ------------------------------------------------------------------------------------------------
# one single-layer configuration (1..4)

def measure_layer(cfg, args, ev, *, steps, warmup, top_level):
    """Everything reported for one single-layer configuration.  Returns a dict."""
    import numpy as np
    import torch
    import paper_2407_15891_amd as razor
    from paper_2407_15891_amd.workloads import make_workload

    dev = "cuda:0"
    lib = razor.load_library()
    stream = torch.cuda.current_stream().cuda_stream
    w0 = make_workload(cfg, dev, materialize=False)
    esize = 4 if w0.dtype == torch.float32 else 2
    out_dtype = w0.dtype                                  # O in the dtype of the inputs
    # enough distinct caches that >= 1 GB of other data goes by between two visits to the same bytes,
    # so the 256 MB memory-side cache cannot serve a step's reads (small configurations stay resident)
    sizes, desc_plan = razor.RazorSizes(), np.zeros(w0.B * w0.Hkv, razor.DESC_DTYPE)
    p0 = razor.RazorParams(w0.B, w0.Hq, w0.Hkv, w0.d, w0.n_sink, w0.window, 0, 1, razor.RAZOR_BF16 if esize == 2 else
                           razor.RAZOR_F32, razor.RAZOR_F32, w0.scale, 0, 0, 0, None, None)
    assert razor.razor_plan(p0, w0.seq_lens, w0.mask, desc_plan, None, sizes) == 0
    one_step = algorithmic_bytes_decode(desc_plan, w0.d, esize, w0.B, w0.Hq, esize)
    copies = min(8, max(args.copies, -(-(1 << 30) // one_step)))
    cache_resident = copies * one_step < (1 << 30)
    total_steps = steps + warmup
    max_new = 4 * (total_steps // copies + 4)             # timed pass, event pass, kernel pass (+ graph warm-up)
    w = make_workload(cfg, dev, max_new=max_new)

    extra = {}
    if args.alibi and top_level:
        w.n_sink = 0
        slopes = (2.0 ** (-8.0 * np.arange(1, w.Hq + 1) / w.Hq)).astype(np.float32)
        extra = dict(use_comp=False, alibi_slopes=torch.from_numpy(slopes).to(dev))
    sliding = bool(args.sliding and top_level)

    def new_cache(mask):
        return razor.RazorCache(batch=w.B, n_q_heads=w.Hq, n_kv_heads=w.Hkv, head_dim=w.d, seq_lens=w.seq_lens,
                                retrieval_mask=mask, n_sink=w.n_sink, window=w.window, max_new=max_new,
                                dtype=w.dtype, out_dtype=out_dtype, scale=w.scale, n_workers=args.workers,
                                device=dev, sliding=sliding, **extra)

    def build_caches(mask, n):
        caches = []
        for _ in range(n):
            c = new_cache(mask)
            c.compress(w.K, w.V)
            caches.append(c)
        torch.cuda.synchronize()
        return caches

    inputs = [w.step_inputs(t) for t in range(8)]       # drawn ahead of the timed region, reused round-robin
    out = torch.empty(w.B, w.Hq, w.d, dtype=out_dtype, device=dev)

    def run_graph(caches, n):
        """n decode steps as replays of one captured graph (one step per cache)."""
        Q, k, v = inputs[0]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            caches[0].decode(Q, k, v, out=out)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for c in caches:
                c.decode(Q, k, v, out=out)
        reps = max(1, n // len(caches))
        g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            g.replay()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * n / (reps * len(caches))

    def run(caches, n, mode="wall"):
        """n decode steps.  mode "wall": wall seconds; "events": per-step GPU ms between a pair of
        events around each call; "kernel": per-step ms of the streaming kernel alone (library hook)."""
        if mode == "wall" and args.graph and top_level:
            return run_graph(caches, n)
        pairs = []
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(n):
            c = caches[t % len(caches)]
            Q, k, v = inputs[t % len(inputs)]
            if mode != "wall":
                a, b = ev.create(), ev.create()
                pairs.append((a, b))
            if mode == "kernel":
                lib.razor_profile_events(a, b)
            elif mode == "events":
                ev.record(a, stream)
            c.decode(Q, k, v, out=out)
            if mode == "events":
                ev.record(b, stream)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        if mode == "wall":
            return dt
        lib.razor_profile_events(None, None)
        ms = [ev.elapsed_ms(a, b) for a, b in pairs]
        for a, b in pairs:
            ev.destroy(a, b)
        return ms

    # ---------------- compressed cache
    caches = build_caches(w.mask, copies)
    desc0 = caches[0].desc()
    run(caches, warmup)
    wall = run(caches, steps)
    step_ms = run(caches, steps, "events")
    kernel_ms = run(caches, steps, "kernel")
    ms_per_step = wall / steps * 1e3
    # rows grow by one per visit; take the table at the middle of the timed region
    desc_avg = desc0.copy()
    desc_avg["rows"] = desc0["rows"] + warmup // copies + steps // (2 * copies)
    if sliding:   # window heads stay at n_sink + window rows
        stay = (desc0["flags"] & razor.RAZOR_HEAD_RETRIEVAL) == 0
        desc_avg["rows"][stay] = np.minimum(desc_avg["rows"][stay], w.n_sink + w.window)
    step_bytes = algorithmic_bytes_decode(desc_avg, w.d, esize, w.B, w.Hq, esize, use_comp=not extra)
    gbps = step_bytes / (wall / steps) / 1e9
    step_us, kernel_us = stats_us(step_ms), stats_us(kernel_ms)
    kernel_gbps = step_bytes / (kernel_us["mean"] * 1e-6) / 1e9
    kept_rows = int(desc0["rows"].astype("int64").sum())
    full_rows = int(w.seq_lens.astype("int64").sum()) * w.Hkv

    # ---------------- what a kernel that only reads gets here
    ceiling = None
    if top_level and not args.no_ceiling:
        ceiling = read_stream_ceiling(ev, stream, int(step_bytes), args.workers)
        ceiling["kernel_frac_of_own_pattern"] = kernel_gbps / ceiling["patterns"]["contiguous"]["GBps"]
        ceiling["kernel_frac_of_best_pattern"] = kernel_gbps / ceiling["best"]["GBps"]

    # ---------------- compression pass
    compress = measure_compress(w, caches, new_cache, desc0, esize, ev, stream, full=top_level)
    del caches
    torch.cuda.empty_cache()

    # ---------------- the same kernels on the uncompressed cache
    full = None
    if not args.no_full:
        fcaches = build_caches(np.ones(w.Hkv, np.uint8), max(2, min(copies, 4) // 2))
        fdesc = fcaches[0].desc()
        n_full = max(10, steps // 4)
        run(fcaches, max(2, warmup // 4))
        fwall = run(fcaches, n_full)
        f_us = stats_us(run(fcaches, n_full, "events"))
        fk_us = stats_us(run(fcaches, n_full, "kernel"))
        fbytes = algorithmic_bytes_decode(fdesc, w.d, esize, w.B, w.Hq, esize)
        full = {"ms_per_step": fwall / n_full * 1e3, "GBps": fbytes / (fwall / n_full) / 1e9, "step_us": f_us,
                "kernel_us": fk_us, "kernel_GBps": fbytes / (fk_us["mean"] * 1e-6) / 1e9, "bytes": fbytes,
                "steps": n_full}
        del fcaches
        torch.cuda.empty_cache()

    # ---------------- CPU oracle on the host cores (reported baseline, not the target)
    cpu = None
    if not args.no_cpu_baseline:
        cpu = oracle_baseline(w, inputs[0], desc0, esize, budget_s=10.0 if top_level else 2.0, new_cache=new_cache)

    byte_ratio = (full["bytes"] / step_bytes) if full else full_rows / kept_rows
    workload = (f"benchmark configuration {cfg}: {w.name}, batch {w.B}, {w.Hq} query / {w.Hkv} KV heads, head_dim "
                f"{w.d}, context {w.N}" + (f" (ragged {int(w.seq_lens.min())}..{int(w.seq_lens.max())})" if cfg == 4 else "")
                + f", window {w.window}, {w.n_sink} sinks, {int(w.mask.sum())} retrieval KV heads; one step = append one "
                "token + compressed decode attention + combine" + (" (sliding mode)" if sliding else "")
                + (" (ALiBi logits, no sinks, no compensation token)" if extra else ""))
    traffic, traffic_file = committed_traffic(cfg)
    return {
        "workload": workload, "cached_rows": kept_rows, "full_rows": full_rows, "copies_rotated": copies,
        "cache_resident": cache_resident, "steps": steps, "warmup": warmup,
        "dtype": "bf16" if w.dtype == torch.bfloat16 else "f32", "out_dtype": "bf16" if out_dtype == torch.bfloat16 else "f32",
        "GBps": gbps, "ms_per_step": ms_per_step, "pct_of_hbm_peak": 100.0 * gbps / HBM_PEAK_GBPS,
        "step_us": step_us, "step_GBps_median": step_bytes / (step_us["median"] * 1e-6) / 1e9,
        "step_frac_of_peak_median": step_bytes / (step_us["median"] * 1e-6) / 1e9 / HBM_PEAK_GBPS,
        "step_bytes": step_bytes, "byte_ratio_full_over_compressed": byte_ratio,
        "speedup_vs_full_cache": (full["ms_per_step"] / ms_per_step) if full else None,
        "speedup_vs_full_cache_gpu_time": (full["step_us"]["median"] / step_us["median"]) if full else None,
        "full_cache": full, "compress": compress,
        "roofline": {"bound": "hbm", "kernel": "decode_partial (streams K/V, online softmax)",
                     "achieved": kernel_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": kernel_gbps / HBM_PEAK_GBPS, "kernel_ms": kernel_us["mean"] * 1e-3,
                     "kernel_us": kernel_us, "traffic": traffic,
                     "traffic_source": (f"{traffic_file}: rocprofv3 FETCH_SIZE + WRITE_SIZE of an earlier run of this "
                                        "command, not measured in this run") if traffic else None,
                     "read_stream_ceiling": ceiling},
        "cpu_baseline": cpu,
    }


def read_stream_ceiling(ev, stream, step_bytes, workers):
    """The library's read-stream probe over as many bytes as one step moves, launches rotating through
    a 4 GiB buffer, for several ways of handing the bytes to the wavefronts."""
    import torch
    import paper_2407_15891_amd as razor
    dev = "cuda:0"
    buf = torch.empty(4 << 30, dtype=torch.uint8, device=dev)
    buf.fill_(1)
    sink = torch.empty(4 * razor.RAZOR_MAX_WORKERS, dtype=torch.uint8, device=dev)

    def probe(nbytes, reps, pattern, depth, nt):
        nbytes = nbytes // 4096 * 4096
        slots = max(1, buf.numel() // nbytes)
        times = []
        a0, b0 = ev.create(), ev.create()
        for r in range(reps + 2):
            addr = buf.data_ptr() + (r % slots) * nbytes
            ev.record(a0, stream)
            rc = razor.razor_probe_read_stream(addr, nbytes, workers, pattern, depth, nt, sink, stream)
            assert rc == 0, razor.razor_strerror(rc)
            ev.record(b0, stream)
            ms = ev.elapsed_ms(a0, b0)
            if r >= 2:
                times.append(ms)
        ev.destroy(a0, b0)
        return {"GBps": nbytes / (sum(times) / len(times) * 1e-3) / 1e9, "GBps_best": nbytes / (min(times) * 1e-3) / 1e9}
    patterns = {"contiguous": probe(step_bytes, 12, razor.RAZOR_PROBE_CONTIGUOUS, 2, 1),
                "interleaved_4KB": probe(step_bytes, 12, razor.RAZOR_PROBE_INTERLEAVED, 2, 1),
                "interleaved_128KB": probe(step_bytes, 12, 32, 2, 1),
                "contiguous_4_in_flight": probe(step_bytes, 12, razor.RAZOR_PROBE_CONTIGUOUS, 4, 1),
                "contiguous_plain_loads": probe(step_bytes, 6, razor.RAZOR_PROBE_CONTIGUOUS, 2, 0)}
    best = max(patterns, key=lambda k: patterns[k]["GBps"])
    whole = probe(4 << 30, 4, razor.RAZOR_PROBE_CONTIGUOUS, 2, 1)
    del buf, sink
    torch.cuda.empty_cache()
    return {"patterns": patterns, "best": {"pattern": best, "GBps": patterns[best]["GBps"]},
            "GBps_4GiB_contiguous": whole["GBps"],
            "how": "razor_probe_read_stream: 128-bit loads in 4 KB wave-wide pieces, one wavefront per SIMD, two "
                   "pieces in flight and non-temporal unless named otherwise; contiguous = one range per wavefront "
                   "(what decode_partial does), interleaved = wavefront w takes every W-th piece / 32-piece chunk; "
                   "events around every launch, mean (and best) of the repetitions on as many bytes as one decode "
                   "step moves, consecutive launches on different parts of a 4 GiB buffer"}


def measure_compress(w, caches, new_cache, desc0, esize, ev, stream, full):
    """The compression pass: repeated on buffers that earlier calls already went through (warm),
    one-shot (K and V rewritten right before, as after a prefill kernel; fresh arena, table and
    workspace every time), and -- `full` only -- given column sums."""
    import torch
    comp_bytes = algorithmic_bytes_compress(desc0, w.seq_lens, w.Hkv, w.d, esize)
    kept_rows = int(desc0["rows"].astype("int64").sum())
    full_rows = int(w.seq_lens.astype("int64").sum()) * w.Hkv
    a, b = ev.create(), ev.create()

    def timed(fn):
        torch.cuda.synchronize()
        ev.record(a, stream)
        fn()
        ev.record(b, stream)
        return ev.elapsed_ms(a, b)

    def rate(us):
        return {"us": us, "GBps": comp_bytes / (us["median"] * 1e-6) / 1e9,
                "pct_of_hbm_peak": 100.0 * comp_bytes / (us["median"] * 1e-6) / 1e9 / HBM_PEAK_GBPS}
    caches[0].compress(w.K, w.V)
    warm = stats_us([timed(lambda: caches[r % len(caches)].compress(w.K, w.V)) for r in range(7)])
    shots = []
    for r in range(5):
        w.K.mul_(1.0)                                        # same bits, freshly written
        w.V.mul_(1.0)
        c = new_cache(w.mask)
        shots.append(timed(lambda: c.compress(w.K, w.V)))
        del c
    one_shot = rate(stats_us(shots))
    # the call also pays for writing back what the producer of K and V left dirty in the 256 MB
    # memory-side cache (whoever reads those lines first does): HBM bytes of the call including that
    inherited = min(256 << 20, 2 * full_rows * w.d * esize)
    one_shot["GBps_with_inherited_writeback"] = (comp_bytes + inherited) / (one_shot["us"]["median"] * 1e-6) / 1e9
    one_shot["pct_of_hbm_peak_with_inherited_writeback"] = 100.0 * one_shot["GBps_with_inherited_writeback"] / HBM_PEAK_GBPS
    res = {"bytes": comp_bytes, "warm": rate(warm), "one_shot": one_shot,
           "ms": warm["median"] * 1e-3, "GBps": comp_bytes / (warm["median"] * 1e-6) / 1e9,
           "pct_of_hbm_peak": 100.0 * comp_bytes / (warm["median"] * 1e-6) / 1e9 / HBM_PEAK_GBPS,
           "note": "each figure is one razor_compress call between a pair of events after a device synchronisation, "
                   "median of the repetitions; one_shot: K and V rewritten in place right before the call (the state a "
                   "prefill kernel leaves: its last 256 MB are still dirty in the memory-side cache and are written back "
                   "to HBM inside this call, whichever kernel reads them first; the *_with_inherited_writeback figures "
                   "count those bytes too), cache buffers allocated for that call"}
    if full:
        # the same pass when the column sums over the sequence come with K and V (a prefill epilogue
        # has them for free): only the kept rows are read and written
        sums = caches[0].column_sums(w.K, w.V)
        colsum = stats_us([timed(lambda: caches[r % len(caches)].column_sums(w.K, w.V)) for r in range(5)])
        caches[0].compress(w.K, w.V, col_sums=sums)
        given = stats_us([timed(lambda: caches[r % len(caches)].compress(w.K, w.V, col_sums=sums)) for r in range(5)])
        given_bytes = 2 * kept_rows * 2 * w.d * esize + 2 * desc0.size * 2 * w.d * 4
        colsum_bytes = full_rows * 2 * w.d * esize + desc0.size * 2 * w.d * 4
        res["given_column_sums"] = {"us": given, "bytes": given_bytes,
                                    "GBps": given_bytes / (given["median"] * 1e-6) / 1e9}
        res["column_sums_pass"] = {"us": colsum, "bytes": colsum_bytes,
                                   "GBps": colsum_bytes / (colsum["median"] * 1e-6) / 1e9}
        del sums
    ev.destroy(a, b)
    return res


def oracle_baseline(w, step_input, desc0, esize, budget_s, new_cache=None):
    """The fp64 oracle's decode of one whole step of the workload, on the host cores; with
    `new_cache` also the error of the library's fp32 output for that step against it."""
    import numpy as np
    import torch
    import paper_2407_15891_amd as razor
    from oracle import razor_oracle as orc
    nb = w.B
    Kc, Vc = w.K[:nb].cpu(), w.V[:nb].cpu()
    oc = orc.OracleCache(Kc, Vc, w.seq_lens[:nb], w.mask, w.n_sink, w.window, max_new=1)
    Q, k, v = step_input
    oc.append(k[:nb].cpu(), v[:nb].cpu())
    Qc = Q[:nb].cpu()
    best, reps, spent = float("inf"), 0, 0.0
    while reps < 3 or (spent < budget_s and reps < 50):
        t0 = time.perf_counter()
        oc.decode(Qc, w.scale)
        dt = time.perf_counter() - t0
        best, reps, spent = min(best, dt), reps + 1, spent + dt
    d_s = desc0[: nb * w.Hkv].copy()
    d_s["rows"] += 1
    sample_bytes = algorithmic_bytes_decode(d_s, w.d, esize, nb, w.Hq, esize)
    parity = None
    if new_cache is not None:      # the same step through the library, written out as fp32
        ref = oc.decode(Qc, w.scale)
        c = new_cache(w.mask)
        c.compress(w.K, w.V)
        c.params.out_dtype = razor.RAZOR_F32
        got = torch.empty(w.B, w.Hq, w.d, dtype=torch.float32, device=Q.device)
        c.decode(Q, k, v, out=got)
        got = got.cpu().numpy().astype(np.float64)
        parity = {"max_abs": float(np.abs(got - ref).max()),
                  "row_relative_max": float((np.linalg.norm(got - ref, axis=-1) /
                                             np.maximum(np.linalg.norm(ref, axis=-1), 1e-30)).max()),
                  "bar": "max-abs <= 2e-3 and row-relative <= 1e-2 on the fp32 output of this step"}
        del c
    return {"value": sample_bytes / best / 1e9, "unit": "GB/s", "cores": int(oc.threads), "kind": "oracle",
            "seconds": best, "parity_of_this_step": parity,
            "sample": f"one full decode step of the workload ({nb} sequences x {w.Hkv} KV heads, "
                      f"{int(d_s['rows'].sum())} cached rows, {w.Hq} query heads), fp64 C + OpenMP oracle, best of "
                      f"{reps} repetitions; building the oracle's cache (Eq.(4) over the dropped rows) is not timed"}


# ------------------------------------------------------------------------------------------------
# configuration 5: the 32-layer stack

def measure_stack(args, ev, *, steps, warmup, full_steps, cpu_baseline):
    """benchmark configuration 5: a 32-layer 8B-shaped stack (GQA 32/8 x 128, bf16), batch 8, context
    131072; per-layer seeded retrieval masks (38 of 256 (layer, KV head) pairs).  Compress every
    layer right after its synthetic prefill (each call is one-shot: K and V just written, fresh
    arena), then `steps` decode steps, each one razor_decode_attn per layer with an append.  The
    full-cache run uses the same kernels with every head retrieval.  Returns a dict, or a dict with
    "skipped" when the device has too little free memory."""
    import numpy as np
    import torch
    import paper_2407_15891_amd as razor
    from paper_2407_15891_amd.workloads import make_workload

    dev = "cuda:0"
    L = args.layers
    lib = razor.load_library()
    stream = torch.cuda.current_stream().cuda_stream
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    need = L * (1.25e9 + (4.4e9 if full_steps else 0)) + 12e9     # arenas (+ full arenas) + one layer's K, V + slack
    if free < need:
        return {"skipped": f"needs about {need / 1e9:.0f} GB of device memory for {L} resident layers, "
                           f"{free / 1e9:.0f} GB free"}
    max_new = 2 * (steps + warmup) + 12                   # timed, event and kernel passes
    caches, fulls, masks = [], [], []
    compress_ms, comp_bytes = [], 0
    a, b = ev.create(), ev.create()
    w = None
    oracle_src = None
    for layer in range(L):
        w = make_workload(5, dev, layer=layer, max_new=max_new)
        masks.append(w.mask.copy())
        c = razor.RazorCache.from_workload(w, n_workers=args.workers, out_dtype=w.dtype)
        torch.cuda.synchronize()
        ev.record(a, stream)
        c.compress(w.K, w.V)
        ev.record(b, stream)
        compress_ms.append(ev.elapsed_ms(a, b))
        comp_bytes += algorithmic_bytes_compress(c.desc_host, w.seq_lens, w.Hkv, w.d, 2)
        caches.append(c)
        if full_steps:
            f = razor.RazorCache(batch=w.B, n_q_heads=w.Hq, n_kv_heads=w.Hkv, head_dim=w.d,
                                 seq_lens=w.seq_lens, retrieval_mask=np.ones(w.Hkv, np.uint8),
                                 n_sink=w.n_sink, window=w.window, max_new=2 * full_steps + warmup + 2,
                                 dtype=w.dtype, out_dtype=w.dtype, scale=w.scale, n_workers=args.workers, device=dev)
            f.compress(w.K, w.V)
            fulls.append(f)
        if layer == 0 and cpu_baseline:
            oracle_src = (w.K.cpu(), w.V.cpu(), w.mask.copy())
        w.K = w.V = None
        if layer % 8 == 7:
            log(f"configuration 5: {layer + 1} of {L} layers compressed")
    torch.cuda.synchronize()
    inputs = [w.step_inputs(t) for t in range(4)]
    out = torch.empty(w.B, w.Hq, w.d, dtype=w.dtype, device=dev)

    def run(stack, n, mode="wall"):
        pairs = []
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(n):
            Q, k, v = inputs[t % len(inputs)]
            if mode == "events":
                s0, s1 = ev.create(), ev.create()
                pairs.append((s0, s1))
                ev.record(s0, stream)
            for c in stack:
                if mode == "kernel":
                    s0, s1 = ev.create(), ev.create()
                    pairs.append((s0, s1))
                    lib.razor_profile_events(s0, s1)
                c.decode(Q, k, v, out=out)
            if mode == "events":
                ev.record(s1, stream)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        if mode == "wall":
            return dt
        lib.razor_profile_events(None, None)
        ms = [ev.elapsed_ms(x, y) for x, y in pairs]
        for x, y in pairs:
            ev.destroy(x, y)
        return ms

    run(caches, warmup)
    wall = run(caches, steps)
    step_us = stats_us(run(caches, max(2, steps // 2), "events"))
    kernel_us = stats_us(run(caches, max(2, min(steps, 8)), "kernel"))   # one entry per (step, layer)
    appended = warmup + steps // 2
    layer_bytes = [algorithmic_bytes_decode(c.desc_host, w.d, 2, w.B, w.Hq, 2) + appended * w.B * w.Hkv * 2 * w.d * 2
                   for c in caches]
    step_bytes = sum(layer_bytes)
    ms_per_step = wall / steps * 1e3
    gbps = step_bytes / (wall / steps) / 1e9
    kernel_gbps = (step_bytes / L) / (kernel_us["mean"] * 1e-6) / 1e9
    full = None
    if full_steps:
        run(fulls, min(warmup, 2))
        fwall = run(fulls, full_steps)
        f_us = stats_us(run(fulls, max(2, full_steps // 2), "events"))
        fbytes = sum(algorithmic_bytes_decode(c.desc_host, w.d, 2, w.B, w.Hq, 2) for c in fulls)
        full = {"ms_per_step": fwall / full_steps * 1e3, "GBps": fbytes / (fwall / full_steps) / 1e9,
                "step_us": f_us, "bytes": fbytes, "steps": full_steps}
    kept_rows = sum(int(c.desc_host["rows"].astype("int64").sum()) for c in caches)
    full_rows = L * w.B * w.Hkv * w.N

    cpu = None
    if oracle_src is not None:
        from oracle import razor_oracle as orc
        Kc, Vc, mask0 = oracle_src
        oc = orc.OracleCache(Kc, Vc, w.seq_lens, mask0, w.n_sink, w.window, max_new=1)
        Q, k, v = inputs[0]
        oc.append(k.cpu(), v.cpu())
        Qc = Q.cpu()
        best, reps, spent = float("inf"), 0, 0.0
        while reps < 3 or (spent < 8.0 and reps < 30):
            t0 = time.perf_counter()
            oc.decode(Qc, w.scale)
            dt = time.perf_counter() - t0
            best, reps, spent = min(best, dt), reps + 1, spent + dt
        d0 = caches[0].desc_host.copy()
        d0["rows"] += 1
        b0 = algorithmic_bytes_decode(d0, w.d, 2, w.B, w.Hq, 2)
        cpu = {"value": b0 / best / 1e9, "unit": "GB/s", "cores": int(oc.threads), "kind": "oracle",
               "seconds_one_layer_step": best,
               "seconds_scaled_to_256_steps_x_32_layers": best * (step_bytes / b0) * 256,
               "sample": f"one full layer-step (layer 0: {w.B} sequences x {w.Hkv} KV heads, {int(d0['rows'].sum())} cached "
                         f"rows, {w.Hq} query heads), fp64 C + OpenMP oracle, best of {reps} repetitions; the 256-step "
                         f"figure scales that time by the bytes of a whole-stack step over this layer's bytes "
                         f"({step_bytes / b0:.1f}, the {L} layers differ in their retrieval heads) and by 256 steps"}
        del oracle_src, oc
    cs = stats_us(compress_ms)
    ev.destroy(a, b)
    result = {
        "workload": f"benchmark configuration 5: {L}-layer 8B-shaped stack, GQA {w.Hq}/{w.Hkv} x {w.d}, batch {w.B}, "
                    f"context {w.N}, window {w.window}, {w.n_sink} sinks, {int(sum(m.sum() for m in masks))} retrieval "
                    f"(layer, KV head) pairs; one step = {L} x (append + compressed decode attention + combine)",
        "cached_rows": kept_rows, "full_rows": full_rows, "steps": steps, "warmup": warmup, "dtype": "bf16",
        "out_dtype": "bf16", "GBps": gbps, "ms_per_step": ms_per_step, "pct_of_hbm_peak": 100.0 * gbps / HBM_PEAK_GBPS,
        "step_us": step_us, "step_GBps_median": step_bytes / (step_us["median"] * 1e-6) / 1e9,
        "step_frac_of_peak_median": step_bytes / (step_us["median"] * 1e-6) / 1e9 / HBM_PEAK_GBPS,
        "step_bytes": step_bytes,
        "byte_ratio_full_over_compressed": (full["bytes"] / step_bytes) if full else full_rows / kept_rows,
        "speedup_vs_full_cache": (full["ms_per_step"] / ms_per_step) if full else None,
        "full_cache": full,
        "end_to_end_attention_s": {"compressed": ms_per_step * 256 / 1e3,
                                   "full_cache": full["ms_per_step"] * 256 / 1e3 if full else None,
                                   "note": "256 decode steps, scaled from the measured steps"},
        "kv_bytes": {"compressed": kept_rows * 512, "full_cache": full_rows * 512},
        "compress": {"ms_all_layers": sum(compress_ms), "bytes": comp_bytes,
                     "GBps": comp_bytes / (sum(compress_ms) * 1e-3) / 1e9,
                     "pct_of_hbm_peak": 100.0 * comp_bytes / (sum(compress_ms) * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "per_layer_us": cs,
                     "note": "every layer's call is one-shot: its K and V were written right before, its arena, table "
                             "and workspace are new"},
        "roofline": {"bound": "hbm", "kernel": "decode_partial (streams K/V, online softmax), one launch per layer",
                     "achieved": kernel_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": kernel_gbps / HBM_PEAK_GBPS,
                     "kernel_ms": kernel_us["mean"] * 1e-3, "kernel_us": kernel_us,
                     "bytes_per_launch_mean": step_bytes / L, "traffic": None},
        "cpu_baseline": cpu,
    }
    del caches, fulls
    torch.cuda.empty_cache()
    return result


# ------------------------------------------------------------------------------------------------
# other modes

def run_head_scores(args, ev):
    """Sec. 3.3 on the paper's prompt size.  One step = every head of --layers layers scored once."""
    import torch
    import paper_2407_15891_amd as razor
    from paper_2407_15891_amd.workloads import make_scoring_workload

    dev = "cuda:0"
    layers = args.layers or 8
    w = make_scoring_workload(dev, n_q_heads=32, n_kv_heads=8, head_dim=128, period=2500, seed=1)
    Q = w.Q.repeat(layers, 1, 1)                     # layers stacked along the head dimension
    K = w.K.repeat(layers, 1, 1)
    Hq, N, d = Q.shape
    stream = torch.cuda.current_stream().cuda_stream
    ws = torch.empty(razor.razor_head_scores_workspace(Hq, N), dtype=torch.uint8, device=dev)
    echo = torch.empty(Hq, dtype=torch.float32, device=dev)
    ind = torch.empty(Hq, dtype=torch.float32, device=dev)

    def step():
        rc = razor.razor_head_scores(Q, K, razor.RAZOR_BF16, Hq, K.shape[0], d, N, Q.stride(0), Q.stride(1),
                                     K.stride(0), K.stride(1), w.scale, w.period, 0, echo, ind, ws, ws.numel(), stream)
        assert rc == 0, razor.razor_strerror(rc)
    steps, warmup = min(args.steps, 20), min(args.warmup, 3)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    a, b = ev.create(), ev.create()
    t0 = time.perf_counter()
    ev.record(a, stream)
    for _ in range(steps):
        step()
    ev.record(b, stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kernel_ms = ev.elapsed_ms(a, b) / steps
    logits = Hq * (N * (N + 1) // 2)                # causal half of Q K^T
    flops = logits * 2 * d                          # multiply + add
    tflops = flops / (kernel_ms * 1e-3) / 1e12
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import razor_oracle as orc
        n_small = 5000                                # the oracle on 16 heads of a 5000-token prompt
        ws_small = make_scoring_workload("cpu", n_q_heads=16, n_kv_heads=4, head_dim=128, period=1250, seed=1)
        t1 = time.perf_counter()
        orc.head_scores(ws_small.Q, ws_small.K, ws_small.scale, ws_small.period)
        dt = time.perf_counter() - t1
        cpu = {"value": 16 * (n_small * (n_small + 1) // 2) * 2 * 128 / dt / 1e12, "unit": "TFLOP/s",
               "cores": min(16, os.cpu_count() or 1), "kind": "oracle",
               "sample": "16 heads x 128 of a 5000-token prompt (period 1250), fp64"}
    print(json.dumps({
        "metric": "head-scoring pass (Sec. 3.3) causal QK^T TFLOP/s", "value": tflops, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": wall / steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"2500 random tokens x 4, {layers} layers of 32/8 heads x 128, one call"},
        "heads_per_s": Hq / (kernel_ms * 1e-3),
        "roofline": {"bound": "mfma", "kernel": "head_scores_kernel<128>", "achieved": tflops, "peak": 2500.0,
                     "unit": "TFLOP/s", "frac": tflops / 2500.0, "kernel_ms": kernel_ms, "traffic": None,
                     # what actually limits the kernel: vector issue slots.  Per logit one fma, one exp2
                     # (two slots) and one add; 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz slots per second
                     # (packed fp32 is not used in this build)
                     "vector_issue": {"slots_per_logit": 4, "achieved_Tslots": logits * 4 / (kernel_ms * 1e-3) / 1e12,
                                      "peak_Tslots": 256 * 4 * 16 * 2.4e9 / 1e12,
                                      "frac": logits * 4 / (kernel_ms * 1e-3) / (256 * 4 * 16 * 2.4e9)}},
        "cpu_baseline": cpu,
    }))


def run_wave_timeline(args):
    """Load balance of the decode streaming kernel: per-wavefront start / located / end times from
    the debug build of the library (`python __graft_entry__.py --timeline` builds
    librazor_timeline.so), which stamps the 100 MHz wall clock in every wave and leaves the stamps
    in the workspace at the offset its razor_timeline_offset() reports.  Prints a text table."""
    import numpy as np
    import torch
    import paper_2407_15891_amd as razor
    from paper_2407_15891_amd.workloads import make_workload

    twin = os.path.join(os.path.dirname(razor.LIB_PATH), "librazor_timeline.so")
    if not os.path.exists(twin):
        sys.exit(f"{twin} not found: run `python __graft_entry__.py --timeline` first")
    assert razor._lib is None, "the product library is already loaded in this process"
    razor.LIB_PATH = twin                       # load the debug twin instead
    lib = razor.load_library()
    lib.razor_timeline_offset.restype = ctypes.c_uint64
    lib.razor_timeline_offset.argtypes = [ctypes.POINTER(razor.RazorParams)]
    W = args.workers or 1024
    assert W <= razor.RAZOR_MAX_WORKERS // 2, "the debug build stamps at most RAZOR_MAX_WORKERS / 2 waves"
    assert args.config != 5, "--wave-timeline takes a single-layer configuration (1..4)"
    w = make_workload(args.config, "cuda:0", max_new=64)
    caches = []
    for _ in range(3):                          # rotate so that no launch finds its cache in the memory-side cache
        c = razor.RazorCache.from_workload(w, n_workers=W)
        c.compress(w.K, w.V)
        caches.append(c)
    Q, k, v = w.step_inputs(0)
    for it in range(12):
        caches[it % 3].decode(Q, k, v)
    torch.cuda.synchronize()
    c = caches[(12 - 1) % 3]
    off = int(lib.razor_timeline_offset(ctypes.byref(c.params)))
    raw = c.workspace[off: off + W * 32].cpu().numpy().view(np.int64).reshape(W, 4)
    desc = c.desc()
    n_heads = w.B * w.Hkv
    total_blocks = int(((desc["rows"] + 15) // 16).sum())
    per = max(2, -(-total_blocks // W))
    active = min(W, -(-total_blocks // per))
    raw = raw[:active]
    us = (raw[:, :3] - raw[:, 0].min()).astype(np.float64) / 100.0
    print(f"config {args.config}: {w.name}; {n_heads} (sequence, KV head) pairs, {total_blocks} blocks, "
          f"{active} waves x {per} blocks")
    for i, name in enumerate(["start", "located", "end"]):
        col = us[:, i]
        print(f"  {name:8s} min {col.min():8.2f}  p50 {np.median(col):8.2f}  p90 {np.percentile(col, 90):8.2f}  "
              f"max {col.max():8.2f} us")
    busy = us[:, 2] - us[:, 0]
    print(f"  wave busy time: mean {busy.mean():.2f} us, max {busy.max():.2f} us, max / mean {busy.max() / busy.mean():.3f}")
    segs = raw[:, 3]
    for s in sorted(set(segs.tolist())):
        sel = segs == s
        print(f"  waves crossing {s} head segment(s): {int(sel.sum()):5d}, end p50 {np.median(us[sel, 2]):7.2f} "
              f"max {us[sel, 2].max():7.2f} us")
    wg = np.arange(active) // 4
    cu_busy = np.array([busy[wg == x].max() for x in range(wg.max() + 1)])
    print(f"  workgroup (= compute unit) busy time: mean {cu_busy.mean():.2f} us, max {cu_busy.max():.2f} us, "
          f"max / mean {cu_busy.max() / cu_busy.mean():.3f}")
    print("  median end per XCD (workgroup id mod 8): " +
          " ".join(f"{np.median(us[(wg % 8) == x, 2]):.1f}" for x in range(8)))


def run_read_stream_sweep(args, ev):
    """What the memory system gives kernels that only move bytes, over the choices the streaming
    kernels make: wavefronts per SIMD x 4 KB pieces in flight x hand-out of pieces x cache hint for a
    read stream of one decode step's size (0.78 GB), and the same for a copy.  Prints a text table."""
    import torch
    import paper_2407_15891_amd as razor
    dev = "cuda:0"
    stream = torch.cuda.current_stream().cuda_stream
    nbytes = 778 * (1 << 20) // 4096 * 4096
    buf = torch.empty(4 << 30, dtype=torch.uint8, device=dev)
    buf.fill_(1)
    dst = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    sink = torch.empty(4 * razor.RAZOR_MAX_WORKERS, dtype=torch.uint8, device=dev)
    slots = buf.numel() // nbytes
    a, b = ev.create(), ev.create()

    def timed(launch, reps=8):
        ts = []
        for r in range(reps + 2):
            addr = buf.data_ptr() + (r % slots) * nbytes
            ev.record(a, stream)
            rc = launch(addr)
            assert rc == 0, razor.razor_strerror(rc)
            ev.record(b, stream)
            ms = ev.elapsed_ms(a, b)
            if r >= 2:
                ts.append(ms)
        ts.sort()
        return nbytes / (ts[len(ts) // 2] * 1e-3) / 1e12
    patterns = [(0, "one contiguous range per wave"), (1, "interleaved, 4 KB pieces"), (32, "interleaved, 128 KB chunks")]
    print(f"read stream, {nbytes / 1e6:.0f} MB per launch, launches rotating through a 4 GiB buffer, TB/s (median of 8)")
    print(f"{'waves/SIMD':>10} {'hand-out':<30} {'hint':<13} " + " ".join(f"{d:>2} in flight" for d in (1, 2, 4, 8)))
    for per_simd in (1, 2, 4):
        for pat, pname in patterns:
            for nt in (1, 0):
                row = [timed(lambda addr: razor.razor_probe_read_stream(addr, nbytes, 1024 * per_simd, pat, depth, nt,
                                                                         sink, stream)) for depth in (1, 2, 4, 8)]
                print(f"{per_simd:>10} {pname:<30} {'non-temporal' if nt else 'plain':<13} " +
                      " ".join(f"{x:11.2f}" for x in row), flush=True)
    print(f"\ncopy, {nbytes / 1e6:.0f} MB read + {nbytes / 1e6:.0f} MB written per launch, two pieces in flight, "
          "TB/s of read + written bytes")
    print(f"{'waves/SIMD':>10} {'hand-out':<30} " + " ".join(f"{h:>18}" for h in ("plain", "nt loads", "nt stores", "nt loads+stores")))
    for per_simd in (1, 2, 4):
        for pat, pname in patterns:
            row = [2 * timed(lambda addr: razor.razor_probe_copy(dst, addr, nbytes, 1024 * per_simd, pat, hints, stream))
                   for hints in range(4)]
            print(f"{per_simd:>10} {pname:<30} " + " ".join(f"{x:18.2f}" for x in row), flush=True)
    ts = []
    for r in range(8):
        src = buf[(r % slots) * nbytes: (r % slots + 1) * nbytes]
        ev.record(a, stream)
        dst.copy_(src)
        ev.record(b, stream)
        ts.append(ev.elapsed_ms(a, b))
    ts.sort()
    print(f"device-to-device copy of the runtime (torch copy_): {2 * nbytes / (ts[len(ts) // 2] * 1e-3) / 1e12:.2f} TB/s")


def run_read_after_write(args, ev):
    """What reading rows costs right after they were written: a 1.4 GiB read stream whose last x MiB were
    filled by a kernel just before (1 GiB of other traffic first, so that earlier launches leave nothing
    behind), for the two ways of handing the stream to the wavefronts.  Prints a text table."""
    import numpy as np
    import torch
    import paper_2407_15891_amd as razor
    dev, MB = "cuda:0", 1 << 20
    stream = torch.cuda.current_stream().cuda_stream
    X = torch.ones(3 << 30, dtype=torch.uint8, device=dev)
    Y = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
    sink = torch.zeros(4 * razor.RAZOR_MAX_WORKERS, dtype=torch.uint8, device=dev)
    n = 1400 * MB
    a, b = ev.create(), ev.create()
    print(f"read stream of {n // MB} MiB (non-temporal 128-bit loads, one wave per SIMD, two 4 KB pieces in flight), us, median of 5")
    print(f"{'last MiB just written':>22} {'interleaved 4 KB pieces':>26} {'one contiguous range per wave':>32}")
    for x in (0, 16, 32, 64, 128, 192, 256, 384, 512, 1024, 1400):
        row = []
        for pattern in (razor.RAZOR_PROBE_INTERLEAVED, razor.RAZOR_PROBE_CONTIGUOUS):
            ts = []
            for r in range(5):
                Y.add_(1)
                Y.add_(1)
                if x:
                    X[n - x * MB: n].fill_(2)
                torch.cuda.synchronize()
                ev.record(a, stream)
                assert razor.razor_probe_read_stream(X, n, 0, pattern, 2, 1, sink, stream) == 0
                ev.record(b, stream)
                ts.append(ev.elapsed_ms(a, b) * 1e3)
            row.append(float(np.median(ts)))
        print(f"{x:>22} {row[0]:>26.1f} {row[1]:>32.1f}", flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--layers", type=int, default=32, help="configuration 5: layers of the stack to build")
    ap.add_argument("--copies", type=int, default=4, help="distinct caches rotated through, so the "
                    "256 MB memory-side cache cannot serve a step's reads from the previous step (raised by "
                    "itself for small configurations, up to 8)")
    ap.add_argument("--workers", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-full", action="store_true", help="skip the uncompressed-cache comparison")
    ap.add_argument("--no-ceiling", action="store_true", help="skip the read-stream ceiling measurement")
    ap.add_argument("--no-other-configs", action="store_true", help="top-level workload only (no other_configs)")
    ap.add_argument("--no-config5", action="store_true", help="leave the 32-layer stack out of other_configs")
    ap.add_argument("--sliding", action="store_true", help="decode in sliding mode (window heads evict "
                    "their oldest row into the compensation token instead of growing)")
    ap.add_argument("--graph", action="store_true", help="time replays of a HIP graph holding one decode "
                    "step per rotated cache (removes host launch overhead; matters for small configs)")
    ap.add_argument("--alibi", action="store_true", help="ALiBi form: Eq.(1) logit bias, no sinks, no "
                    "compensation token, per-head buffer lengths (retrieval heads keep everything)")
    ap.add_argument("--head-scores", action="store_true", help="time the head-scoring pass of Sec. 3.3 instead "
                    "(2500 random tokens x 4, --layers layers of 32/8 heads x 128 stacked in one call); prints "
                    "its own JSON line, bound by the matrix cores")
    ap.add_argument("--wave-timeline", action="store_true", help="per-wave finish times of the decode streaming "
                    "kernel on --config (1..4) from the debug build of the library; prints a text table")
    ap.add_argument("--read-stream-sweep", action="store_true", help="table of what the memory system gives a read "
                    "stream and a copy under the streaming kernels' choices; prints text")
    ap.add_argument("--read-after-write", action="store_true", help="table of what a read stream pays for rows that "
                    "a kernel wrote just before (the state a prefill leaves for the compression pass); prints text")
    ap.add_argument("--pmc-calib", action="store_true", help="also run one plain 1 GiB device copy, the "
                    "known-size kernel that rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); the path would shard by KV head "
              "and batch with no exchange between GPUs", file=sys.stderr)
        sys.exit(2)

    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    ev = HipEvents()

    if args.wave_timeline:
        return run_wave_timeline(args)
    if args.read_stream_sweep:
        return run_read_stream_sweep(args, ev)
    if args.read_after_write:
        return run_read_after_write(args, ev)
    if args.head_scores:
        return run_head_scores(args, ev)

    plain = not (args.sliding or args.alibi or args.graph)
    if args.config == 5:
        top = measure_stack(args, ev, steps=args.steps, warmup=max(1, min(args.warmup, 4)),
                            full_steps=0 if args.no_full else max(2, args.steps // 8),
                            cpu_baseline=not args.no_cpu_baseline)
        if "skipped" in top:
            print("bench.py: configuration 5 " + top["skipped"], file=sys.stderr)
            sys.exit(2)
    else:
        log(f"configuration {args.config}")
        top = measure_layer(args.config, args, ev, steps=args.steps, warmup=args.warmup, top_level=True)

    if args.pmc_calib:   # the known-size kernel counter readings are scaled by
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    others = None
    if plain and not args.no_other_configs and args.config == 3:
        others = {}
        for cfg in (1, 2, 4):
            log(f"other_configs: configuration {cfg}")
            others[f"config{cfg}"] = measure_layer(cfg, args, ev, steps=40, warmup=8, top_level=False)
        if not args.no_config5:
            log("other_configs: configuration 5")
            others["config5"] = measure_stack(args, ev, steps=8, warmup=2, full_steps=0 if args.no_full else 2,
                                              cpu_baseline=not args.no_cpu_baseline)

    result = {
        "metric": METRIC, "value": top["GBps"], "unit": "GB/s", "n_gpus": 1, "steps": top["steps"],
        "warmup": top["warmup"], "ms_per_step": top["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": top["dtype"], "data": "synthetic",
        "config": {"workload": top["workload"], "cached_rows": top["cached_rows"], "full_rows": top["full_rows"],
                   "copies_rotated": top.get("copies_rotated")},
    }
    for key in ("out_dtype", "pct_of_hbm_peak", "step_us", "step_GBps_median", "step_frac_of_peak_median", "step_bytes",
                "byte_ratio_full_over_compressed", "speedup_vs_full_cache", "speedup_vs_full_cache_gpu_time",
                "full_cache", "end_to_end_attention_s", "kv_bytes", "compress", "roofline", "cpu_baseline"):
        if key in top:
            result[key] = top[key]
    if others is not None:
        result["other_configs"] = others
    print(json.dumps(result))


if __name__ == "__main__":
    main()
