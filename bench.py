#!/usr/bin/env python3
"""Benchmark of the multi-Bulyan hot path on one MI355X.

A step = one mbulyan_aggregate call (distance pass, reduction, selection,
coordinate pass) over one synthetic workload resident in HBM.  Prints ONE JSON
line: whole-job GB/s of gradient input, the roofline of the dominant kernel
(the distance pass) from HIP-event timings taken inside the timed region, and
the CPU oracle timed on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--mode selected|alg1]
"""
import argparse
import json
import sys
import time

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
# HBM bytes per launch of the distance kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, each
# scaled by what the same counter reads for a 4 GiB device copy (FETCH_SIZE reads half the bytes
# of the copy, WRITE_SIZE all of them); see profiles/gram_dma_kernel_cfg4_n39_d250M_hbm_traffic.md
MEASURED_TRAFFIC_BYTES = {(4, "f32"): 2 * 19043016 * 1024 + 9216 * 1024,
                          (4, "bf16"): 2 * 9521538 * 1024 + 9216 * 1024,
                          (4, "fp16"): 2 * 9521540 * 1024 + 9216 * 1024,
                          (5, "f32"): 2 * 24924287 * 1024 + 10240 * 1024}
MFMA_FP32_PEAK_TFLOPS = 157.3  # MI355X dense fp32 matrix, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix, published


def paper_protocol(fn, sync):
    """Section V-A: synchronise, start the timer, run, synchronise, stop; 7 runs, drop the 2 furthest
    from the median, mean and standard deviation (ms) of the remaining 5."""
    runs = []
    for _ in range(7):
        sync()
        r0 = time.perf_counter()
        fn()
        sync()
        runs.append((time.perf_counter() - r0) * 1e3)
    med = sorted(runs)[3]
    kept = sorted(runs, key=lambda x: abs(x - med))[:5]
    mean5 = sum(kept) / 5
    return mean5, (sum((x - mean5) ** 2 for x in kept) / 5) ** 0.5


def sweep():
    """The paper's aggregation-time sweep (Section V-A): n in 7, 9, .., 39, d in 1e5, 1e6, 1e7,
    f = floor((n-3)/4), n gradients drawn from U(0,1)^d; multi-Bulyan (both readings), multi-Krum and
    the coordinate-wise median, each timed with the paper's protocol.  One JSON line per (n, d)."""
    import torch
    import paper_1905_04374_amd as mb
    import workloads as W
    dev = "cuda:0"
    sync = torch.cuda.synchronize
    for d in (100_000, 1_000_000, 10_000_000):
        for n in range(7, 40, 2):
            f = (n - 3) // 4
            G = W.uniform(n, d, dev)
            out = torch.empty(d, device=dev)
            ws = torch.empty(mb.mbulyan_workspace_bytes(n, d), dtype=torch.uint8, device=dev)
            row = {"n": n, "f": f, "d": d}
            calls = {
                "multi_bulyan_ms": lambda: mb.mbulyan_aggregate_ex(G, f, out=out, workspace=ws),
                "multi_bulyan_alg1_ms": lambda: mb.mbulyan_aggregate_ex(G, f, mode=mb.MODE_ALG1, out=out, workspace=ws),
                "multi_krum_ms": lambda: mb.multikrum_aggregate(G, f, out=out, workspace=ws),
                "median_ms": lambda: mb.coordwise_median(G, out=out),
            }
            for name, fn in calls.items():
                fn()
                mean5, std5 = paper_protocol(fn, sync)
                row[name] = round(mean5, 4)
                row[name.replace("_ms", "_std")] = round(std5, 4)
            print(json.dumps(row), flush=True)


def host_resident(a, mb, W, n, f, d, mode, dtype):
    """Gradients that stay in (pinned) host memory: every step uploads them (once if they fit the device; twice
    if not, or with --host-two-sweeps: the selection needs the distances over all coordinates before any
    coordinate can be aggregated) and downloads the result."""
    import torch
    mb.mbulyan_host_resident_limit(0 if a.host_two_sweeps else -1)
    uploads = 2 if a.host_two_sweeps else 1
    g = torch.empty(n, d, device="cuda:0", dtype=torch.float32)
    W.fill(a.config, g, 0)
    host = torch.empty(n, d, dtype=dtype, pin_memory=True)
    host.copy_(g)
    del g
    out = torch.empty(d, dtype=torch.float32, pin_memory=True)
    for _ in range(a.warmup):
        mb.mbulyan_aggregate_host(host, f, a.host_resident, mode=mode, host_out=out)
    t0 = time.perf_counter()
    for _ in range(a.steps):
        mb.mbulyan_aggregate_host(host, f, a.host_resident, mode=mode, host_out=out)   # blocks until out is written
    sec = (time.perf_counter() - t0) / a.steps
    eb = host.element_size()
    print(json.dumps({
        "metric": "multi-Bulyan aggregation GB/s of gradient input, gradients in pinned host memory (PCIe-inclusive)",
        "value": round(eb * n * d / sec / 1e9, 2), "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(sec * 1e3, 3), "higher_is_better": True, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"configs[{a.config - 1}] with d={d}: n={n} f={f} {a.input_dtype}, mode={a.mode}, host-resident, "
                               f"chunks of {a.host_resident} coordinates, uploaded {'twice' if uploads == 2 else 'once'}"},
        "pcie_bytes_per_step": int(uploads * eb * n * d + 4 * d),
        "pcie_GBps": round((uploads * eb * n * d + 4 * d) / sec / 1e9, 2)}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--sweep", action="store_true", help="run the paper's (n, d) sweep on U(0,1) inputs instead")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, help="workload 1..5 (default: the one the metric is quoted on)")
    ap.add_argument("--d", type=int, default=None, help="override the number of coordinates")
    ap.add_argument("--mode", choices=["selected", "alg1"], default="selected")
    ap.add_argument("--dist-algo", choices=["auto", "direct", "gram", "gram_bf16"], default="auto")
    ap.add_argument("--input-dtype", choices=["f32", "bf16", "fp16"], default="f32",
                    help="bf16 / fp16: the workload rounded to that format once, aggregated by the entry points "
                         "for 16-bit storage (half the bytes; a second workload, not the headline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="also run one plain device copy of this many MiB before the timed region "
                         "(a kernel of known traffic, to scale rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--cpu-sample", type=int, default=1 << 28, help="coordinates the oracle is timed on")
    ap.add_argument("--host-resident", type=int, default=0, metavar="CHUNK_D",
                    help="time mbulyan_aggregate_host instead: the workload in pinned HOST memory, uploaded twice in "
                         "column chunks of CHUNK_D coordinates (a PCIe-inclusive rate: a line of its own, never the "
                         "headline value)")
    ap.add_argument("--host-two-sweeps", action="store_true",
                    help="with --host-resident: force the path of a matrix beyond the device (two uploads) although "
                         "this one fits and would be uploaded once")
    a = ap.parse_args()
    if a.sweep:
        return sweep()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the aggregation rule of one parameter server); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    import paper_1905_04374_amd as mb
    import workloads as W

    dev = "cuda:0"
    mb.mbulyan_set_dist_algo({"auto": mb.DIST_AUTO, "direct": mb.DIST_DIRECT, "gram": mb.DIST_GRAM,
                              "gram_bf16": mb.DIST_GRAM_BF16}[a.dist_algo])
    spec = W.spec(a.config)
    n, f = spec["n"], spec["f"]
    d = a.d or spec["d"]
    nchunks = spec["chunks"] if a.d is None else 1
    mode = mb.MODE_SELECTED if a.mode == "selected" else mb.MODE_ALG1
    theta, beta = mb.mbulyan_params(n, f, mode)
    in16 = a.input_dtype in ("bf16", "fp16")
    dt16 = torch.bfloat16 if a.input_dtype == "bf16" else torch.float16
    eb = 2.0 if in16 else 4.0

    if a.host_resident:
        return host_resident(a, mb, W, n, f, d, mode, dt16 if in16 else torch.float32)

    # ---- inputs resident in HBM before the timed region ----------------------
    bounds = [d * k // nchunks for k in range(nchunks + 1)]
    chunks = []
    for k in range(nchunks):
        g = torch.empty(n, bounds[k + 1] - bounds[k], device=dev, dtype=torch.float32)
        W.fill(a.config, g, bounds[k])
        if in16:
            g16 = torch.empty(g.shape, device=dev, dtype=dt16)
            for r in range(n):                     # row by row: no second fp32-sized temporary
                g16[r].copy_(g[r])
            g = g16
        chunks.append(g)
    outs = [torch.empty(c.shape[1], device=dev, dtype=torch.float32) for c in chunks]
    sel = torch.empty(theta, device=dev, dtype=torch.int32)
    ws = torch.empty(mb.mbulyan_workspace_bytes(n, max(c.shape[1] for c in chunks)), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()

    def step():
        if nchunks == 1:
            mb.mbulyan_aggregate_ex(chunks[0], f, mode=mode, out=outs[0], selected_idx=sel, workspace=ws)
        else:
            mb.mbulyan_aggregate_chunked(chunks, f, mode=mode, outs=outs, selected_idx=sel, workspace=ws)

    if a.copy_calibration:
        src = torch.ones(a.copy_calibration << 18, device=dev, dtype=torch.float32)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    # the timed region carries HIP events around the dominant kernel only (two records per launch);
    # events around every stage would cost the small workloads tens of microseconds per step
    mb.mbulyan_timing_reset()
    mb.mbulyan_timing_enable(True, stages=("dist",))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    mb.mbulyan_timing_enable(False)
    dominant = mb.mbulyan_timing_read()["dist"]
    # per-stage split: the same steps once more, every stage between events (not part of `value`)
    mb.mbulyan_timing_reset()
    mb.mbulyan_timing_enable(True)
    for _ in range(a.steps):
        step()
    torch.cuda.synchronize()
    mb.mbulyan_timing_enable(False)
    stages = mb.mbulyan_timing_read()

    mean5, std5 = paper_protocol(step, torch.cuda.synchronize)

    sec = (t1 - t0) / a.steps
    in_bytes = eb * n * d
    # rows the coordinate pass reads: the theta extracted ones, or (Algorithm-1 reading) the rows of the first
    # round's averaged set, n-f-2 of them, which holds every later set while the score order stays stable
    rows2 = theta if mode == mb.MODE_SELECTED else n - f - 2
    value = in_bytes / sec / 1e9

    # dominant kernel: the distance pass, 4*n bytes per coordinate, one launch per chunk
    dist_ms, dist_launches = dominant
    dist_avg_s = dist_ms / 1e3 / max(dist_launches, 1)
    dist_bytes = in_bytes / nchunks
    achieved = dist_bytes / dist_avg_s / 1e9
    bf16 = a.dist_algo in ("auto", "gram_bf16")
    nb = (n + 15) // 16
    # rows that start on 16-byte boundaries take the kernel that streams tiles into LDS
    gram = "gram_dma_kernel" if (d // nchunks) % 4 == 0 and d // nchunks >= 128 else "gram_kernel"
    kname = {"direct": "dist_direct_kernel", "gram": f"{gram}<{nb}, fp32>"}.get(
        a.dist_algo, f"{gram}<{nb}, bf16>")
    if in16:
        kname = f"gram_dma_kernel<{nb}, {a.input_dtype} input>"
    roofline = {"kernel": kname, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": MEASURED_TRAFFIC_BYTES.get((a.config, a.input_dtype))
                if (bf16 and a.d is None) else None,
                "algorithmic_bytes": dist_bytes,
                "avg_launch_ms": round(dist_avg_s * 1e3, 4), "launches": dist_launches}
    if a.dist_algo != "direct":
        # matrix-core work of the same kernel: lower block triangle of 16x16 tiles, one (fp32) or six
        # (split bf16) products per tile and coordinate
        tiles = nb * (nb + 1) // 2
        flops = tiles * 256 * 2 * (1 if in16 else 6 if bf16 else 1) * (d / nchunks)
        peak = MFMA_BF16_PEAK_TFLOPS if (bf16 or in16) else MFMA_FP32_PEAK_TFLOPS   # bf16 and fp16: the same dense peak
        roofline["matrix_cores"] = {"dtype": a.input_dtype if in16 else "bf16" if bf16 else "f32", "tflops": round(flops / dist_avg_s / 1e12, 1),
                                    "peak": peak, "frac": round(flops / dist_avg_s / 1e12 / peak, 4)}

    per_stage = {k: round(v[0] / a.steps, 4) for k, v in stages.items()}
    coord_ms, coord_launches = stages["coord"]
    if rows2 is not None and coord_launches:
        coord_bytes = (eb * rows2 + 4.0) * d / nchunks
        per_stage["coord_GBps"] = round(coord_bytes / (coord_ms / 1e3 / coord_launches) / 1e9, 1)
        alg_bytes = (eb * (n + rows2) + 4.0) * d
        per_stage["hbm_frac_algorithmic_bytes"] = round(alg_bytes / sec / 1e9 / HBM_PEAK_GBS, 4)

    res = {
        "metric": "multi-Bulyan aggregation GB/s of gradient input (n*d*4B/s), 1 GPU" if not in16 else
                  f"multi-Bulyan aggregation GB/s of gradient input (n*d*2B/s, {a.input_dtype} gradients), 1 GPU",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(sec * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"configs[{a.config - 1}]: n={n} f={f} d={d} {a.input_dtype + ' gradients' if in16 else 'fp32'}, "
                               f"mode={a.mode}, "
                               f"theta={theta} beta={beta}, chunks={nchunks}"},
        "hbm_frac_input_bytes": round(value / HBM_PEAK_GBS, 4),
        "stage_ms_per_step": per_stage,
        "paper_protocol_ms": {"mean_of_5": round(mean5, 4), "std_of_5": round(std5, 4), "runs": 7},
        "roofline": roofline,
    }

    if not a.no_cpu_baseline:
        import oracle as O
        omode = O.MODE_SELECTED if mode == mb.MODE_SELECTED else O.MODE_ALG1
        ds = min(a.cpu_sample, chunks[0].shape[1])
        host = chunks[0][:, :ds].float().contiguous().cpu().numpy()

        def oracle_run(threads):
            """the oracle's three phases, timed one by one (seconds)"""
            c0 = time.perf_counter()
            D = O.pairwise_sqdist(host, nthreads=threads)
            c1 = time.perf_counter()
            ext, sets, _ = O.multikrum_select(D, f, theta)
            c2 = time.perf_counter()
            if omode == O.MODE_SELECTED:
                O.coordwise_selected(host, ext, beta, nthreads=threads)
            else:
                O.coordwise_alg1(host, ext, sets, beta, nthreads=threads)
            c3 = time.perf_counter()
            return c1 - c0, c2 - c1, c3 - c2, O.last_threads()

        t_dist, t_sel, t_coord, cores = oracle_run(0)
        total = t_dist + t_sel + t_coord
        res["cpu_baseline"] = {"value": round(eb * n * ds / total / 1e9, 3), "unit": "GB/s",
                               "cores": cores, "kind": "oracle",
                               "sample": f"first {ds} of {d} coordinates, all {n} rows, whole rule, "
                                         f"{round(total, 2)} s",
                               "phases_s": {"distance": round(t_dist, 4), "selection": round(t_sel, 6),
                                            "coordinate": round(t_coord, 4)}}
        if a.config <= 2:        # small enough for one thread as well
            t1 = oracle_run(1)
            res["cpu_baseline"]["single_thread"] = {
                "value": round(eb * n * ds / sum(t1[:3]) / 1e9, 3), "unit": "GB/s",
                "phases_s": {"distance": round(t1[0], 4), "selection": round(t1[1], 6), "coordinate": round(t1[2], 4)}}
        del host
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
