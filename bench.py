#!/usr/bin/env python3
"""Benchmark of the ZipCCL codec hot path on one MI355X.

A step = one compress + one decompress of the whole workload (all peer chunks), inputs
resident in HBM.  Prints ONE JSON line: round-trip throughput in uncompressed GB/s for the
headline workload (c5, the largest), the per-direction rates and compression ratio, the HBM
roofline of the dominant kernel measured live with events on the launch stream, the CPU oracle
timed on the host cores, the legs built next to the codec (fused reduce, sigma estimates), and the
same codec figures for every other workload (`other_workloads`).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5] [--no-others] [--no-cpu]
"""
import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0            # MI355X HBM3E, published peak
KERNELS = {"compress": "zipccl_compress = k_compress + k_place (one call, two launches; chunks of more than 4096 tiles add k_tile_scan)",
           "decompress": "zipccl_decompress = k_decompress"}
PAPER_CONTEXT = ("paper (64x RTX A6000, 200 Gb/s): communication time -1.35x, end-to-end training 1.18x; "
                 "it prints no codec GB/s, so vs_baseline is null")
OTHERS = ("c3", "c4", "c5", "c5_fp32", "c2", "c1")
CACHE_RESIDENT = ("c1", "c2")      # 2 MiB and 32 MiB: they fit the 256 MB last-level cache and are launch-bound


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


SETTLE_S = 0.08     # load the chip this long before timing: see warm_up()


def warm_up(step, warmup):
    """Untimed steps: at least `warmup` of them and at least SETTLE_S of uninterrupted load.  When load starts
    after an idle spell (an allocation, a check on the host) the chip runs ~2 ms at its top clock, then slows down
    for some 20 ms (a kernel bound by instruction issue by up to 40 %, one waiting on memory by ~5 %) and
    recovers; the timed steps follow the warm-up without a gap, so they see the steady state.
    Returns the number of steps run."""
    import torch
    done = 0
    t0 = time.perf_counter()
    while done < max(1, warmup) or time.perf_counter() - t0 < SETTLE_S:
        for _ in range(5):
            step()
        done += 5
        torch.cuda.synchronize()
    return done


def frac(nbytes, ms):
    return round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)


def run_gpu(w, steps, warmup):
    import torch
    import paper_2604_27844_amd.binding as z
    from paper_2604_27844_amd.yardstick import zipccl_yardstick_copy

    dev = torch.device("cuda:0")
    signed = np.int16 if w.dtype == z.BF16 else np.int32
    d_in = torch.from_numpy(w.data.view(signed)).to(dev)
    table = z.zipccl_build_table(w.sigma, w.dtype)
    cap = z.zipccl_max_compressed_size(w.n_elems, w.dtype, w.n_chunks, w.chunk_elems)
    d_out = torch.empty(cap, dtype=torch.uint8, device=dev)
    d_cb = torch.zeros(w.n_chunks, dtype=torch.int64, device=dev)
    d_ws = torch.empty(z.zipccl_compress_workspace_size(w.n_elems, w.dtype, w.n_chunks, w.chunk_elems),
                       dtype=torch.uint8, device=dev)
    d_back = torch.empty_like(d_in)
    d_st = torch.zeros(1, dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream()

    def compress():
        z.zipccl_compress(d_in, w.n_elems, w.dtype, w.n_chunks, w.chunk_elems, table, d_out, d_cb, d_ws, stream=stream)

    def decompress():
        z.zipccl_decompress(d_out, d_back, w.n_elems, w.dtype, w.n_chunks, w.chunk_elems, d_st, stream=stream)

    compress()
    decompress()
    torch.cuda.synchronize()
    assert int(d_st.item()) == 0
    assert torch.equal(d_back, d_in), "round trip is not the identity"
    comp_bytes = int(d_cb.sum().item())

    # W untimed steps, then K timed ones, bracketed by synchronize; events (on the launch stream) split the directions
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    warm = warm_up(lambda: (compress(), decompress()), warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        evs[k][0].record(stream)
        compress()
        evs[k][1].record(stream)
        decompress()
        evs[k][2].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    tc = np.array([e[0].elapsed_time(e[1]) for e in evs])      # ms
    td = np.array([e[1].elapsed_time(e[2]) for e in evs])

    # yardstick: a plain copy kernel moving the same number of bytes as one codec launch
    # ((nbytes + comp_bytes) / 2 read and as many written)
    half = min((w.nbytes + comp_bytes) // 2, w.nbytes) // 16 * 16
    cevs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(5)]
    for k in range(5):
        cevs[k][0].record(stream)
        zipccl_yardstick_copy(d_back, d_in, half, stream=stream)
        cevs[k][1].record(stream)
    torch.cuda.synchronize()
    copy_ms = float(np.median([e[0].elapsed_time(e[1]) for e in cevs]))
    return dict(wall_s=wall, tc_ms=tc, td_ms=td, comp_bytes=comp_bytes, copy_GBps=2 * half / (copy_ms * 1e-3) / 1e9,
                d_in=d_in, d_out=d_out, d_cb=d_cb, d_ws=d_ws, table=table, warm=warm)


def run_reduce(w, peers, steps):
    """The first widening beyond the codec: decode `peers` received slices and sum them in FP32
    (zipccl_decompress_reduce).  The workload is cut into `peers` equal slices standing for the
    peers' contributions to one shard."""
    import torch
    import paper_2604_27844_amd.binding as z
    if w.n_elems % peers:
        return None
    dev = torch.device("cuda:0")
    n = w.n_elems // peers
    bf16 = w.dtype == z.BF16
    d_in = torch.from_numpy(w.data.view(np.int16 if bf16 else np.int32)).to(dev)
    as_f32 = (lambda t: t.view(torch.bfloat16).float()) if bf16 else (lambda t: t.view(torch.float32))
    table = z.zipccl_build_table(w.sigma, w.dtype)
    cap = z.zipccl_max_compressed_size(w.n_elems, w.dtype, peers)
    d_comp = torch.empty(cap, dtype=torch.uint8, device=dev)
    d_cb = torch.zeros(peers, dtype=torch.int64, device=dev)
    d_ws = torch.empty(z.zipccl_compress_workspace_size(w.n_elems, w.dtype, peers), dtype=torch.uint8, device=dev)
    z.zipccl_compress(d_in, w.n_elems, w.dtype, peers, None, table, d_comp, d_cb, d_ws)
    d_sum = torch.empty(n, dtype=torch.float32, device=dev)
    d_st = torch.zeros(1, dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream()
    z.zipccl_decompress_reduce(d_comp, d_sum, n, w.dtype, peers, z.FP32, d_st, stream=stream)
    torch.cuda.synchronize()
    assert int(d_st.item()) == 0
    ref = as_f32(d_in[:n]).clone()
    for p in range(1, peers):
        ref = ref + as_f32(d_in[p * n:(p + 1) * n])
    assert torch.equal(ref.view(torch.int32), d_sum.view(torch.int32)), "fused reduce differs from peer-ordered FP32 sum"
    del ref
    d_sum16 = torch.empty(n, dtype=torch.int16, device=dev)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(steps)]
    evs16 = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(steps)]
    warm_up(lambda: z.zipccl_decompress_reduce(d_comp, d_sum, n, w.dtype, peers, z.FP32, d_st, stream=stream), 5)
    for k in range(steps):
        evs[k][0].record(stream)
        z.zipccl_decompress_reduce(d_comp, d_sum, n, w.dtype, peers, z.FP32, d_st, stream=stream)
        evs[k][1].record(stream)
    torch.cuda.synchronize()
    ts = [e[0].elapsed_time(e[1]) for e in evs]
    ms, ms_min = float(np.median(ts)), float(min(ts))
    # the same sums rounded to bf16 (what a gradient shard kept in bf16 would receive)
    for k in range(steps):
        evs16[k][0].record(stream)
        z.zipccl_decompress_reduce(d_comp, d_sum16, n, w.dtype, peers, z.BF16, d_st, stream=stream)
        evs16[k][1].record(stream)
    torch.cuda.synchronize()
    ts = [e[0].elapsed_time(e[1]) for e in evs16]
    ms16, ms16_min = float(np.median(ts)), float(min(ts))
    assert torch.equal(d_sum16.view(torch.bfloat16), d_sum.to(torch.bfloat16)), "bf16 output is not the rounded FP32 sum"
    comp_bytes = int(d_cb.sum().item())
    algo = comp_bytes + 4 * n
    return {"peers": peers, "n_per_peer": n, "ms": round(ms, 4), "ms_min": round(ms_min, 4), "ms_bf16_out": round(ms16, 4),
            "ms_bf16_out_min": round(ms16_min, 4),
            "timing": "calls back to back after 80 ms of the same load: median and fastest",
            "hbm_frac_bf16_out": frac(comp_bytes + 2 * n, ms16),
            "uncompressed_in_GBps": round(w.nbytes / (ms * 1e-3) / 1e9, 1),
            "algorithmic_bytes": algo, "hbm_GBps": round(algo / (ms * 1e-3) / 1e9, 1),
            "hbm_frac": frac(algo, ms),
            "checked": "bit-equal to the peer-ordered FP32 sum of the inputs"}


def run_estimate(w, r, steps):
    """sigma / table from the data on the device, one read of the tensor each: the sample standard deviation
    (zipccl_estimate_table, what section 4.1 names) and the median-based sigma (zipccl_estimate_table_robust);
    and the compression ratio each table gives on this workload next to the nominal-sigma table's.
    steps = 0: no timing."""
    import torch
    import paper_2604_27844_amd.binding as z
    dev = torch.device("cuda:0")
    d_in, d_out, d_cb, d_ws = r["d_in"], r["d_out"], r["d_cb"], r["d_ws"]
    d_tab = torch.zeros(8, dtype=torch.uint8, device=dev)
    d_sig = torch.zeros(1, dtype=torch.float64, device=dev)
    stream = torch.cuda.current_stream()
    out = {"ratio_with_nominal_sigma_table": round(w.nbytes / r["comp_bytes"], 5), "nominal_sigma": w.sigma,
           "nominal_dec1": int(r["table"].dec[1])}
    legs = (("sample_std", z.zipccl_estimate_table, z.zipccl_estimate_workspace_size()),
            ("robust_median", z.zipccl_estimate_table_robust, z.zipccl_estimate_robust_workspace_size()))
    for name, fn, ws_bytes in legs:
        d_ews = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        call = lambda: fn(d_in, w.n_elems, w.dtype, d_tab, d_sig, d_ews, stream=stream)
        leg = {}
        if steps:
            evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(steps)]
            warm_up(call, 1)
            for k in range(steps):
                evs[k][0].record(stream)
                call()
                evs[k][1].record(stream)
            torch.cuda.synchronize()
            ts = [e[0].elapsed_time(e[1]) for e in evs]
            ms = float(np.median(ts))
            leg.update({"ms": round(ms, 4), "ms_min": round(float(min(ts)), 4),
                        "hbm_GBps": round(w.nbytes / (ms * 1e-3) / 1e9, 1), "hbm_frac": frac(w.nbytes, ms)})
        else:
            call()
        z.zipccl_compress_device_table(d_in, w.n_elems, w.dtype, w.n_chunks, w.chunk_elems, d_tab, d_out, d_cb, d_ws,
                                       stream=stream)
        torch.cuda.synchronize()
        leg.update({"sigma": float(d_sig.item()), "dec1": int(d_tab[1].item()),
                    "ratio_with_estimated_table": round(w.nbytes / int(d_cb.sum().item()), 5)})
        out[name] = leg
    # one robust table per peer chunk (zipccl_estimate_chunk_tables + zipccl_compress_chunk_tables)
    d_tabs = torch.zeros(8 * w.n_chunks, dtype=torch.uint8, device=dev)
    d_ews = torch.empty(z.zipccl_estimate_chunk_tables_workspace_size(w.n_chunks), dtype=torch.uint8, device=dev)
    call = lambda: z.zipccl_estimate_chunk_tables(d_in, w.n_elems, w.dtype, w.n_chunks, w.chunk_elems, d_tabs, None, d_ews,
                                                  stream=stream)
    leg = {}
    if steps:
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(steps)]
        warm_up(call, 1)
        for k in range(steps):
            evs[k][0].record(stream)
            call()
            evs[k][1].record(stream)
        torch.cuda.synchronize()
        ts = [e[0].elapsed_time(e[1]) for e in evs]
        ms = float(np.median(ts))
        leg.update({"ms": round(ms, 4), "ms_min": round(float(min(ts)), 4), "hbm_frac": frac(w.nbytes, ms)})
    else:
        call()
    z.zipccl_compress_chunk_tables(d_in, w.n_elems, w.dtype, w.n_chunks, w.chunk_elems, d_tabs, d_out, d_cb, d_ws, stream=stream)
    torch.cuda.synchronize()
    dec1 = d_tabs.view(-1, 8)[:, 1].cpu().numpy()
    leg.update({"dec1_min": int(dec1.min()), "dec1_max": int(dec1.max()),
                "ratio_with_estimated_tables": round(w.nbytes / int(d_cb.sum().item()), 5)})
    out["robust_median_per_chunk"] = leg
    # the same per-chunk tables from one group of 512 values in every 16 (zipccl_estimate_chunk_tables_sampled)
    SAMPLE = 16
    d_tabs_s = torch.zeros(8 * w.n_chunks, dtype=torch.uint8, device=dev)
    call = lambda: z.zipccl_estimate_chunk_tables_sampled(d_in, w.n_elems, w.dtype, w.n_chunks, w.chunk_elems, SAMPLE,
                                                          d_tabs_s, None, d_ews, stream=stream)
    leg = {"sample_stride": SAMPLE}
    if steps:
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(steps)]
        warm_up(call, 1)
        for k in range(steps):
            evs[k][0].record(stream)
            call()
            evs[k][1].record(stream)
        torch.cuda.synchronize()
        ts = [e[0].elapsed_time(e[1]) for e in evs]
        leg.update({"ms": round(float(np.median(ts)), 4), "ms_min": round(float(min(ts)), 4)})
    else:
        call()
    z.zipccl_compress_chunk_tables(d_in, w.n_elems, w.dtype, w.n_chunks, w.chunk_elems, d_tabs_s, d_out, d_cb, d_ws, stream=stream)
    torch.cuda.synchronize()
    leg.update({"tables_equal_to_the_full_estimate": bool(torch.equal(d_tabs_s, d_tabs)),
                "ratio_with_estimated_tables": round(w.nbytes / int(d_cb.sum().item()), 5)})
    out["robust_median_per_chunk_sampled"] = leg
    return out


def run_oracle(w, gpu_out=None, gpu_cb=None, parallel=True):
    """The oracle as it stands: single thread over the whole workload, then one chunk per host thread."""
    import oracle
    dec = oracle.build_table(w.sigma)
    t0 = time.perf_counter()
    ref, ref_cb, off = oracle.compress(w.data, w.dtype, dec, w.n_chunks, w.chunk_elems)
    t1 = time.perf_counter()
    back = oracle.decompress(ref, w.n_elems, w.dtype, w.n_chunks, w.chunk_elems)
    t2 = time.perf_counter()
    assert np.array_equal(back, w.data)
    same = None
    if gpu_out is not None:
        same = bool(np.array_equal(gpu_cb, ref_cb))
        for c in range(0, w.n_chunks, max(1, w.n_chunks // 8)):    # sampled slots, byte for byte
            s, e = int(off[c]), int(off[c]) + int(ref_cb[c])
            same = same and bool(np.array_equal(gpu_out[s:e], ref[s:e]))
    gb = w.nbytes / 1e9
    cores = len(os.sched_getaffinity(0))
    res = dict(single=dict(compress_GBps=gb / (t1 - t0), decompress_GBps=gb / (t2 - t1), roundtrip_GBps=gb / (t2 - t0)),
               ratio=w.nbytes / float(ref_cb.sum()), matches_gpu=same, host_cores=cores)
    if parallel:
        # chunk-parallel: every peer slice is independent
        ce = w.chunk_elems if w.chunk_elems is not None else np.full(w.n_chunks, w.n_elems // w.n_chunks, dtype=np.uint64)
        starts = np.concatenate([[0], np.cumsum(ce)]).astype(np.int64)

        def one(c):
            x = w.data[starts[c]:starts[c + 1]]
            o, cb, _ = oracle.compress(x, w.dtype, dec)
            oracle.decompress(o, x.size, w.dtype)

        threads = min(cores, w.n_chunks)
        t3 = time.perf_counter()
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(one, range(w.n_chunks)))
        t4 = time.perf_counter()
        res["parallel"] = dict(roundtrip_GBps=gb / (t4 - t3), threads=threads)
    return res


def codec_entry(w, r, with_oracle):
    """The per-workload figures of `other_workloads`: both directions, median and fastest call, against that
    workload's own algorithmic bytes."""
    tc, td = float(np.median(r["tc_ms"])), float(np.median(r["td_ms"]))
    ab = w.nbytes + r["comp_bytes"]
    e = {"MiB": round(w.nbytes / 2**20, 1), "n_chunks": w.n_chunks, "ragged": w.chunk_elems is not None,
         "dtype": "u16" if w.dtype == 0 else "u32",
         "compress_ms": round(tc, 4), "compress_ms_min": round(float(r["tc_ms"].min()), 4),
         "decompress_ms": round(td, 4), "decompress_ms_min": round(float(r["td_ms"].min()), 4),
         "compress_GBps": round(w.nbytes / 1e9 / (tc * 1e-3), 2), "decompress_GBps": round(w.nbytes / 1e9 / (td * 1e-3), 2),
         "algorithmic_bytes_per_call": ab, "compress_frac": frac(ab, tc), "decompress_frac": frac(ab, td),
         "copy_kernel_frac": round(r["copy_GBps"] / HBM_PEAK_GBPS, 4),
         "compression_ratio": round(w.nbytes / r["comp_bytes"], 5)}
    if with_oracle:
        o = run_oracle(w, r["d_out"].cpu().numpy(), r["d_cb"].cpu().numpy().astype(np.uint64), parallel=False)
        e.update({"gpu_bytes_match_oracle": o["matches_gpu"], "oracle_ratio": round(o["ratio"], 5),
                  "oracle_1thread_roundtrip_GBps": round(o["single"]["roundtrip_GBps"], 4)})
    return e


def main():
    global SETTLE_S
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=20)   # at least; warm_up() also loads the chip for --settle-ms
    ap.add_argument("--settle-ms", type=float, default=SETTLE_S * 1e3, help="minimum duration of every warm-up (counter runs: 0)")
    ap.add_argument("--workload", default="c5", help="c1|c2|c3|c4|c5|c5_fp32 (default: c5, the largest)")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (parity/debug only)")
    ap.add_argument("--no-others", action="store_true", help="only the headline workload (profiling runs)")
    ap.add_argument("--all", action="store_true", help="accepted for compatibility: every workload is timed by default")
    ap.add_argument("--no-cpu", action="store_true", help="skip every oracle leg")
    ap.add_argument("--chunks", type=int, default=0, help="override the workload's chunk count with an equal split")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is a single-GPU codec path; run with --gpus 1 "
                 "(no collective or second GPU is used anywhere)")

    import torch
    from paper_2604_27844_amd import workloads
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU (the product path has no CPU fallback)")

    log(f"generating workload {args.workload} (scale {args.scale})")
    w = workloads.make(args.workload, args.scale)
    if args.chunks:
        w.n_chunks, w.chunk_elems = args.chunks, None
    log(f"{w.name}: n={w.n_elems} ({w.nbytes / 2**20:.0f} MiB), {w.n_chunks} chunks, sigma={w.sigma}")
    SETTLE_S = args.settle_ms * 1e-3
    r = run_gpu(w, args.steps, args.warmup)
    gb = w.nbytes / 1e9
    tc, td = float(r["tc_ms"].mean()), float(r["td_ms"].mean())
    tc_med, td_med = float(np.median(r["tc_ms"])), float(np.median(r["td_ms"]))
    ms_per_step = r["wall_s"] * 1e3 / args.steps
    algo_bytes = w.nbytes + r["comp_bytes"]       # each direction reads one side and writes the other
    dominant = "compress" if tc >= td else "decompress"
    t_dom = max(tc, td)
    achieved = algo_bytes / (t_dom * 1e-3) / 1e9
    es = 2 if w.dtype == 0 else 4
    traffic = None
    tfile = os.path.join(ROOT, "profiles", "hbm_traffic.json")     # from the rocprofv3 --pmc runs summarised beside it
    if os.path.exists(tfile):
        traffic = json.load(open(tfile)).get(f"{args.workload}:{dominant}")

    out = {
        "metric": "codec_roundtrip_uncompressed_GBps", "value": round(gb / (ms_per_step * 1e-3), 2), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "warmup_run": r["warm"], "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u16" if w.dtype == 0 else "u32", "data": "synthetic",
        "config": {"workload": w.name, "n_elems": w.n_elems, "elem_bytes": es, "n_chunks": w.n_chunks,
                   "ragged": w.chunk_elems is not None, "table_sigma": w.sigma, "group": 512, "scale": args.scale},
        "compress_GBps": round(gb / (tc_med * 1e-3), 2), "decompress_GBps": round(gb / (td_med * 1e-3), 2),
        "compress_ms": round(tc_med, 4), "decompress_ms": round(td_med, 4),
        "compress_ms_mean": round(tc, 4), "decompress_ms_mean": round(td, 4),
        "compress_ms_min": round(float(r["tc_ms"].min()), 4), "decompress_ms_min": round(float(r["td_ms"].min()), 4),
        "timing": "event-timed calls on the launch stream; *_ms = median of the timed steps, *_ms_mean their mean, *_ms_min the fastest",
        "compression_ratio": round(w.nbytes / r["comp_bytes"], 5),
        "roofline": {"bound": "hbm", "kernel": KERNELS[dominant], "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "achieved_from": "algorithmic bytes per call / mean event-timed duration of the slower call",
                     "traffic": traffic,
                     "traffic_source": "profiles/hbm_traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run "
                                       "of this command, summarised in profiles/; not measured in this run)",
                     "algorithmic_bytes_per_launch": algo_bytes,
                     "compress_frac": frac(algo_bytes, tc), "decompress_frac": frac(algo_bytes, td),
                     "compress_frac_median": frac(algo_bytes, tc_med), "decompress_frac_median": frac(algo_bytes, td_med),
                     "copy_kernel_GBps": round(r["copy_GBps"], 1)},
        "paper_context": PAPER_CONTEXT,
    }

    if not args.no_cpu:
        log("timing the CPU oracle on the same workload")
        o = run_oracle(w, r["d_out"].cpu().numpy(), r["d_cb"].cpu().numpy().astype(np.uint64))
        out["cpu_baseline"] = {"value": round(o["single"]["roundtrip_GBps"], 4), "unit": "GB/s", "cores": 1,
                               "kind": "oracle",
                               "sample": f"the whole workload ({w.nbytes / 2**20:.0f} MiB), compress + decompress, "
                                         "scalar C oracle on one host thread",
                               "compress_GBps": round(o["single"]["compress_GBps"], 4),
                               "decompress_GBps": round(o["single"]["decompress_GBps"], 4),
                               "all_cores": {"value": round(o["parallel"]["roundtrip_GBps"], 4),
                                             "cores": o["parallel"]["threads"],
                                             "how": "one peer chunk per host thread"},
                               "host_cores": o["host_cores"], "ratio": round(o["ratio"], 5),
                               "gpu_bytes_match_oracle": o["matches_gpu"]}
    log("sigma estimates")
    out["estimate_table"] = run_estimate(w, r, max(3, args.steps // 2))
    del r
    torch.cuda.empty_cache()
    log("fused reduce")
    red = run_reduce(w, 8, max(3, args.steps))
    if red:
        out["decompress_reduce"] = red

    if not args.no_others:
        extra = {}
        for name in OTHERS:
            if name == args.workload:
                continue
            log(f"workload {name}")
            w2 = workloads.make(name, args.scale)
            r2 = run_gpu(w2, args.steps, args.warmup)
            e = codec_entry(w2, r2, not args.no_cpu)
            if name in CACHE_RESIDENT:
                e["cache_resident"] = True          # launch-bound: outside the >= 256 MB target
            e["estimate_table"] = run_estimate(w2, r2, 0)
            extra[w2.name] = e
            del r2, w2
            torch.cuda.empty_cache()
        out["other_workloads"] = extra
        big = [v for v in extra.values() if not v.get("cache_resident")]
        out["min_frac_over_256MB_workloads"] = min([out["roofline"]["compress_frac_median"], out["roofline"]["decompress_frac_median"]] +
                                                  [x for v in big for x in (v["compress_frac"], v["decompress_frac"])])

    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
