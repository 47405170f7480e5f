#!/usr/bin/env python3
"""Benchmark of the sampling epilogue on one MI355X.

A "step" is one pass of the whole hot path (penalties -> filter -> softmax -> draw, SHVS when
the workload has a hot set) over one batch of synthetic logits that is already resident in HBM.
Default workload: B=1024, V=128,256, fp32, heterogeneous per-row controls, 4096 history ids per
row (the configuration the headline metric is quoted on).  Prints ONE JSON line on stdout.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2|3|4|5] [--H N] [--no-cpu-baseline]
                  [--all-configs]

--all-configs also runs C2, C4 (at each hot-set size of its sweep) and C5 for a few steps and prints
one JSON line per run on stderr; stdout stays the one line of the headline configuration.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0  # MI355X published HBM3E bandwidth


def algorithmic_bytes(B: int, V: int, esize: int, nnz_total: int) -> int:
    """Bytes the method must move per call: every logit once, every history id once, and per row
    the parameter record (32), the CSR offset (8) and the output id (4)."""
    return B * V * esize + 4 * nnz_total + 44 * B


KERNEL_SOURCES = ("simple_fast.hip", "simple_rowdev.hpp", "simple_device.hpp", "simple_kernels.hpp")


def kernel_source_hash() -> str:
    """sha256 over the sources of the dominant kernel: recorded counter readings only hold for the
    kernel they were taken on."""
    import hashlib
    h = hashlib.sha256()
    for f in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2512_00719_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def recorded_traffic(config: int):
    """HBM bytes per launch of the dominant kernel from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs
    summarised under profiles/, or None if there is no summary for this workload or the kernel's
    sources have changed since the counters were taken."""
    path = os.path.join(ROOT, "profiles", f"fast_rows_kernel_C{config}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    fields = {}
    with open(path) as fh:
        for line in fh:
            if ":" in line and not line.startswith("#"):
                k, v = line.split(":", 1)
                fields[k.strip()] = v.strip()
    if fields.get("kernel_source_sha256") != kernel_source_hash():
        return None
    try:
        return int(fields["traffic_bytes_per_launch"])
    except (KeyError, ValueError):
        return None


_CPU_W = None  # the workload, for the forked workers of the all-core leg


def _oracle_rows(span) -> int:
    """Rows [b0, b1) of the workload through the CPU oracle, one by one; returns the row count."""
    from oracle import simple_oracle as O
    w = _CPU_W
    b0, b1 = span
    has_hist = w.hist_ids.size > 0
    hot_mask = O.hot_mask_from_ids(w.hot_ids, w.V)
    for b in range(b0, b1):
        zr = w.logits[b] if w.dtype == "f32" else ((w.logits[b].astype(np.uint32) << np.uint32(16)).view(np.float32))
        hr = w.hist_ids[int(w.hist_ptr[b]):int(w.hist_ptr[b + 1])] if has_hist else None
        O.sample_row(zr, w.params[b], hr, hot_mask, w.seed, b, 0)
    return b1 - b0


def cpu_baseline(w, budget_s: float = 10.0) -> dict:
    """The CPU oracle, as it stands, timed on a bounded sample of rows of the same workload: on one
    core, then the same rows-at-a-time loop on every core this process may use (forked workers, so
    this runs before the process touches the GPU)."""
    global _CPU_W
    _CPU_W = w
    rows_done, t0 = 0, time.perf_counter()
    while rows_done < w.B and time.perf_counter() - t0 < budget_s:
        rows_done += _oracle_rows((rows_done, rows_done + 1))
    dt = time.perf_counter() - t0
    out = {"value": rows_done / dt, "unit": "rows/s", "cores": 1, "kind": "oracle",
           "sample": f"first {rows_done} rows of the workload, one call (step 0), single thread numpy, {dt:.1f} s"}
    try:
        import multiprocessing as mp
        n = max(1, min(16, len(os.sched_getaffinity(0))))
        if n > 1:
            chunk = 4
            want = min(w.B, max(chunk * n, int(out["value"] * n * budget_s * 0.8)))
            spans = [(b, min(b + chunk, want)) for b in range(0, want, chunk)]
            with mp.get_context("fork").Pool(n) as pool:
                t1 = time.perf_counter()
                done = sum(pool.map(_oracle_rows, spans, chunksize=1))
                dt_all = time.perf_counter() - t1
            out["all_cores"] = {"value": done / dt_all, "unit": "rows/s", "cores": n,
                                "sample": f"first {done} rows, {n} forked workers, {dt_all:.1f} s"}
    except (OSError, ValueError) as e:  # no fork on this host: the single-core figure stands alone
        out["all_cores"] = {"value": None, "note": str(e)}
    return out


METRIC = {
    2: "sampled rows/sec + achieved HBM GB/s (fraction of peak), B=256 V=151,936 bf16",
    3: "sampled rows/sec + achieved HBM GB/s (fraction of peak), B=1024 V=128,256 fp32",
    4: "sampled rows/sec + achieved HBM GB/s (fraction of peak), B=512 V=201,088 bf16, SHVS",
    5: "sampled rows/sec + achieved HBM GB/s (fraction of peak), B=4096 V=256,000 bf16, SHVS H=16,384",
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--H", type=int, default=None, help="hot-set size for configs 4 and 5")
    ap.add_argument("--copies", type=int, default=0, help="distinct input copies to rotate over (0 = auto: >= 1 GiB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stateful", action="store_true",
                    help="take the rows' histories from an incremental penalty state (simple_sample_state) instead of the CSR arrays")
    ap.add_argument("--hot-first-sweep", action="store_true",
                    help="instead of the headline run: SHVS on a hot-first vocabulary with caller-supplied tail statistics "
                         "(simple_sample_hot_first), swept over the hot-set size, with the paper's sizing model on the result")
    ap.add_argument("--all-configs", action="store_true", help="also run C2, C4 (H sweep) and C5 briefly; their lines go to stderr")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="after the timed region, run one plain device copy of this many MiB (a kernel of known "
                         "HBM traffic, to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(rows are independent: N GPUs would each take B / N rows and call it unchanged)", file=sys.stderr)
        return 2

    if args.hot_first_sweep:
        return hot_first_sweep(args)
    result = run_config(args, args.config, args.H, args.steps, args.warmup, not args.no_cpu_baseline)
    if args.all_configs:
        sweep = []
        for cfg, H in ((2, None), (4, 4096), (4, 8192), (4, 16384), (4, 32768), (5, None)):
            if cfg == args.config and H == args.H:
                continue
            r = run_config(args, cfg, H, min(args.steps, 50), min(args.warmup, 10), False)
            print(json.dumps(r), file=sys.stderr, flush=True)
            if cfg == 4:
                sweep.append((H, r["ms_per_step"] * 1e-3 / 512, r["config"]["shvs_mean_alpha"]))
        if len(sweep) >= 2:
            # the paper's sizing model (section 5.4) on the measured sweep: cost per row against H, hit ratio, F(H);
            # reference constants: the affine CPU fit the paper reports for its own samplers
            from paper_2512_00719_amd import sizing
            print(json.dumps({"sizing_C4": sizing.summarize_sweep([h for h, _, _ in sweep], [t for _, t, _ in sweep],
                                                                  [a for _, _, a in sweep], 201_088, reference=(1.06e-8, 8.55e-6))}),
                  file=sys.stderr, flush=True)
    print(json.dumps(result), flush=True)
    return 0


def hot_first_sweep(args) -> int:
    """The GPU analogue of the paper's sizing experiment (section 7, sizing model validation): rows that
    sample with temperature alone on a hot-first vocabulary of C4's shape, a batch large enough that
    the time per call reflects the average cost of a row (accepted rows read H columns, rejected ones
    their tail as well).  Per H: the measured cost per row, the hot path's own cost (every draw forced
    to accept by statistics that declare an empty tail), acceptance and mean alpha; then the affine fit
    T(H) = c H + c0 of the hot path, F(H) of Eq. (cpu-time) and its minimiser against the measured one."""
    import torch
    from paper_2512_00719_amd import binding, sizing, synth
    B, V = 4096, 201_088
    rng = np.random.default_rng(synth.DATA_SEED_BASE + 6)
    logits_np = synth.zipf_profile_logits(B, V, 1.2, 1.0, rng, "bf16", np.arange(V, dtype=np.int64))
    dev = "cuda:0"
    lg = torch.from_numpy(logits_np.view(np.int16)).to(dev).view(torch.bfloat16)
    par = synth.make_params(B, temperature=1.0)
    params = torch.from_numpy(par.view(np.uint8).reshape(B, 32)).to(dev)
    out = torch.empty(B, dtype=torch.int32, device=dev)
    s = binding.Sampler(V, 0, max_B=B)
    stats_dev = torch.zeros(64, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    rows = []
    for H in ((args.H,) if args.H else (2048, 4096, 8192, 16384, 32768, 65536)):
        # what the producer of the logits would supply (temperature 1): maximum and exponential sum of each row's tail
        tail = lg[:, H:].float()
        tmax = tail.max(dim=1).values
        tsum = torch.exp((tail - tmax[:, None]).double()).sum(dim=1)
        ts = np.zeros(B, binding.TAIL_STATS_DTYPE)
        ts["tail_max"] = tmax.cpu().numpy(); ts["tail_sum"] = tsum.cpu().numpy()
        del tail
        real = torch.from_numpy(ts.view(np.uint8).reshape(B, 16)).to(dev)
        ts_none = ts.copy(); ts_none["tail_sum"] = 0.0    # an empty tail: every draw is accepted (timing of the hot path alone)
        forced = torch.from_numpy(ts_none.view(np.uint8).reshape(B, 16)).to(dev)

        def run(tsd, n):
            for i in range(n):
                rc = binding.simple_sample_hot_first(s.ctx, lg.data_ptr(), B, V, binding.SIMPLE_BF16, lg.stride(0), params.data_ptr(), H,
                                                     tsd.data_ptr(), synth.SAMPLER_SEED, i, 0, out.data_ptr(), 0, stream)
                assert rc == 0, rc
        times = {}
        for name, tsd in (("measured", real), ("hot_path", forced)):
            run(tsd, 5)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            run(tsd, args.steps if args.steps < 200 else 50)
            torch.cuda.synchronize()
            times[name] = (time.perf_counter() - t0) / (args.steps if args.steps < 200 else 50)
        stats_dev.zero_()
        assert binding.simple_set_stats(s.ctx, stats_dev.data_ptr()) == 0
        run(real, 1)
        torch.cuda.synchronize()
        assert binding.simple_set_stats(s.ctx, 0) == 0
        agg = stats_dev.cpu().numpy().view(binding.STATS_DTYPE)[0]
        n = int(agg["shvs_accepted"] + agg["shvs_rejected"])
        row = {"H": H, "ms_per_call": times["measured"] * 1e3, "ms_per_call_hot_path_only": times["hot_path"] * 1e3,
               "rows_per_s": B / times["measured"], "acceptance_rate": float(agg["shvs_accepted"]) / n,
               "mean_alpha": float(agg["sum_alpha_q32"]) / 2.0 ** 32 / n,
               "bytes_read_per_row_model": (float(agg["shvs_accepted"]) * H + float(agg["shvs_rejected"]) * V) * 2 / n}
        rows.append(row)
        print(json.dumps({"hot_first": row}), file=sys.stderr, flush=True)
    Hs = [r["H"] for r in rows]
    if len(rows) < 2:  # a single hot-set size (--H): no fit
        print(json.dumps({"sweep": rows}), flush=True)
        s.close()
        return 0
    c, c0 = sizing.fit_affine_cost(Hs, [r["ms_per_call_hot_path_only"] * 1e-3 / B for r in rows])
    alpha = [r["mean_alpha"] for r in rows]
    F = sizing.expected_cost(Hs, alpha, c, c0, V)
    measured = [r["ms_per_call"] * 1e-3 / B for r in rows]
    summary = {"workload": f"hot-first sweep: B={B} V={V} bf16, Zipf(1.2) profile + N(0,1) noise in rank order, temperature 1, no truncation",
               "hot_path_fit": {"c_seconds_per_column": c, "c0_seconds": c0},
               "F_model_seconds_per_row": [float(x) for x in F], "measured_seconds_per_row": measured,
               "best_H_model": Hs[int(np.argmin(F))], "best_H_measured": Hs[int(np.argmin(measured))], "sweep": rows}
    print(json.dumps(summary), flush=True)
    s.close()
    return 0


def run_config(args, config: int, H_arg, steps: int, warmup: int, cpu_leg: bool) -> dict:
    import torch
    from paper_2512_00719_amd import binding, synth

    t_gen = time.perf_counter()
    w = synth.make_config(config, H=H_arg)
    esize = 4 if w.dtype == "f32" else 2
    nnz_total = int(w.hist_ids.size)
    nnz_max = int(np.diff(w.hist_ptr).max()) if nnz_total else 0
    alg_bytes = algorithmic_bytes(w.B, w.V, esize, nnz_total)
    print(f"[bench] {w.name}: B={w.B} V={w.V} {w.dtype} nnz/row={nnz_max} "
          f"algorithmic bytes/call={alg_bytes / 1e6:.1f} MB (generated in {time.perf_counter() - t_gen:.1f} s)",
          file=sys.stderr, flush=True)

    # the CPU leg forks workers: it runs before this process initialises the GPU
    cpu = cpu_baseline(w) if cpu_leg else None
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    # Rotate over distinct copies of the inputs so that the 256 MB memory-side cache cannot serve
    # repeated reads: at least 1 GiB is touched between two uses of the same copy.
    n_copies = args.copies or max(2, int(np.ceil((1 << 30) / (w.B * w.V * esize))))
    if w.dtype == "f32":
        host = torch.from_numpy(w.logits)
    else:
        host = torch.from_numpy(w.logits.view(np.int16)).view(torch.bfloat16)
    logits = [host.to(dev) for _ in range(n_copies)]
    params = torch.from_numpy(w.params.view(np.uint8).reshape(w.B, 32)).to(dev)
    hist_ptr = torch.from_numpy(w.hist_ptr).to(dev) if nnz_total else None
    hist_ids = [torch.from_numpy(w.hist_ids).to(dev) for _ in range(n_copies)] if nnz_total else [None] * n_copies
    hot_ids = torch.from_numpy(w.hot_ids).to(dev) if w.hot_ids is not None else None
    out = torch.empty(w.B, dtype=torch.int32, device=dev)
    diag = torch.zeros(w.B * 32, dtype=torch.uint8, device=dev)

    s = binding.Sampler(w.V, nnz_max, max_B=w.B)
    stats_dev = torch.zeros(64, dtype=torch.uint8, device=dev)
    H = 0
    if hot_ids is not None:  # the bitmap is built once, outside the timed region
        s.set_hot_set(hot_ids, w.V)
        H = -1

    state = None
    if args.stateful and nnz_total:
        # every sequence's tokens so far are loaded as generated tokens (n_prompt = 0, as in the CSR form of the workload)
        state = binding.simple_state_create(0, w.B, w.V, nnz_max)
        zeros = torch.zeros(w.B, dtype=torch.int32, device=dev)
        rc = binding.simple_state_restart(state, 0, w.B, hist_ptr.data_ptr(), hist_ids[0].data_ptr(), zeros.data_ptr(),
                                          torch.cuda.current_stream().cuda_stream)
        assert rc == 0, rc
        ref = s.sample(logits[0], params, hist_ptr, hist_ids[0], None, H, seed=w.seed, step=0, V=w.V).clone()

    def step(i: int, with_diag: bool = False):
        c = i % n_copies
        if state is not None:
            rc = binding.simple_sample_state(s.ctx, state, 0, logits[c].data_ptr(), w.B, w.V, dt_code, logits[c].stride(0),
                                             params.data_ptr(), 0, H, w.seed, i, 0, out.data_ptr(),
                                             diag.data_ptr() if with_diag else 0, torch.cuda.current_stream().cuda_stream)
            assert rc == 0, rc
            return
        s.sample(logits[c], params, hist_ptr, hist_ids[c], None, H, seed=w.seed, step=i, out=out,
                 diag=diag if with_diag else None, V=w.V)

    dt_code = binding.SIMPLE_F32 if w.dtype == "f32" else binding.SIMPLE_BF16
    if state is not None:
        step(0)
        torch.cuda.synchronize()
        assert torch.equal(out, ref), "stateful and stateless calls disagree"

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    # The library brackets its dominant kernel (the single-pass row kernel) with HIP events on the
    # stream it launches on; the whole step (both kernels of a call) is timed by the wall clock
    # between two device synchronisations.
    timed = min(steps, 1024)
    assert binding.simple_profile_enable(s.ctx, True) == 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(warmup + i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    n_rec, total_ms = binding.simple_profile_read(s.ctx)
    assert n_rec == timed, (n_rec, timed)
    kern_ms = total_ms / n_rec  # average launch duration of the dominant kernel
    per_launch = binding.simple_profile_read_launches(s.ctx)
    p10, p50, p90 = (float(x) for x in np.percentile(per_launch, [10, 50, 90]))
    binding.simple_profile_enable(s.ctx, False)
    ms_per_step = wall * 1e3 / steps
    rows_per_s = w.B * steps / wall

    # one more call, outside the timed region, with the library's device-side aggregate installed
    assert binding.simple_set_stats(s.ctx, stats_dev.data_ptr()) == 0
    step(warmup + steps)
    torch.cuda.synchronize()
    assert binding.simple_set_stats(s.ctx, 0) == 0
    agg = stats_dev.cpu().numpy().view(binding.STATS_DTYPE)[0]
    stats = {"second_pass_rows": int(agg["second_pass_rows"]), "general_kernel_rows": int(agg["general_rows"]),
             "error_flags": int(agg["error_flags"])}
    if hot_ids is not None:
        n_shvs = int(agg["shvs_accepted"] + agg["shvs_rejected"])
        stats["shvs_acceptance_rate"] = float(agg["shvs_accepted"]) / max(n_shvs, 1)
        stats["shvs_mean_alpha"] = float(agg["sum_alpha_q32"]) / 2.0 ** 32 / max(n_shvs, 1)
        stats["H"] = int(w.hot_ids.size)
    achieved = alg_bytes / (kern_ms * 1e-3) / 1e9
    s.close()
    if state is not None:
        binding.simple_state_destroy(state)

    # What a one-pass row kernel can reach here: the library's read-only row-maximum reduction over
    # the same logits copies, timed with events on the stream it is launched on.
    row_max = torch.empty(w.B, dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()
    def probe(i: int):
        lg = logits[i % n_copies]
        rc = binding.simple_stream_probe(lg.data_ptr(), w.B, w.V, dt_code, lg.stride(0), row_max.data_ptr(),
                                         stream.cuda_stream)
        assert rc == 0, rc

    n_probe = 50
    for i in range(5):
        probe(i)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for i in range(n_probe):
        probe(5 + i)
    e1.record(stream)
    e1.synchronize()
    probe_ms = e0.elapsed_time(e1) / n_probe
    ceiling = (w.B * w.V * esize + w.B * 4) / (probe_ms * 1e-3) / 1e9
    if args.copy_probe_mib > 0:
        src = torch.ones(args.copy_probe_mib << 18, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()

    kernel_name = "simple::fast::fast_rows_kernel"
    if config == 4:  # every row is a bfloat16 row without top-k and penalties: the pattern-count kernel completes them all
        kernel_name = "simple::pattern::pattern_rows_kernel (and the launch of simple::fast::fast_rows_kernel behind it, which finds no row)"
    call_gbs = alg_bytes / (ms_per_step * 1e-3) / 1e9
    traffic = recorded_traffic(config)
    result = {
        "metric": METRIC[config],
        "value": rows_per_s, "unit": "rows/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B} V={w.V} {w.dtype} logits (Zipf profile + noise), "
                               f"{nnz_max} history ids/row, heterogeneous per-row controls"
                               if config in (3, 5) else f"{w.name}: B={w.B} V={w.V} {w.dtype}, {nnz_max} history ids/row",
                   "input_copies_rotated": n_copies, "history": "incremental state" if state is not None else "CSR arrays", **stats},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": achieved / PEAK_HBM_GBS, "traffic": traffic,
                     "traffic_source": None if traffic is None else "recorded: rocprofv3 counter runs summarised under profiles/, "
                                                                    "valid while the kernel's sources are unchanged",
                     "kernel": kernel_name, "kernel_ms": kern_ms,
                     "kernel_ms_p10_p50_p90": [p10, p50, p90], "algorithmic_bytes": alg_bytes,
                     "stream_ceiling": {"what": "read-only row-maximum reduction over the same logits",
                                        "ms": probe_ms, "achieved": ceiling, "frac_of_peak": ceiling / PEAK_HBM_GBS},
                     "frac_of_stream_ceiling": achieved / ceiling,
                     # every kernel of the call (the dominant one, the kernels behind it, the gaps between them)
                     "whole_call": {"ms": ms_per_step, "achieved": call_gbs, "frac": call_gbs / PEAK_HBM_GBS}},
    }
    if cpu is not None:
        result["cpu_baseline"] = cpu
    del logits, hist_ids
    torch.cuda.empty_cache()
    return result


if __name__ == "__main__":
    sys.exit(main())
